// Two-dimensional LSTM layer (Sec. 4.2 of the RETURNN paper): the hidden state of pixel (u, v)
// needs the states of (u-1, v) and (u, v-1) in scan order, so all pixels of one anti-diagonal can
// be computed together; four scan directions and several images run at once.
//
// One workgroup per (scan direction, image, band of 16 rows); it walks the
// anti-diagonals on which its band has pixels, at the image's own width, so images of a batch never
// wait for each other.  A band needs one row of its neighbouring band per diagonal; that dependency
// runs one way (see "rows handed between the bands" below), so the neighbour runs ahead.  In scan
// coordinates (row r = 0 .. Hh-1, column q = 0 .. width-1) diagonal s holds the pixels r + q = s;
// the pixel of row r on diagonal s has its vertical predecessor in row r-1 and its horizontal
// predecessor in row r, both on diagonal s-1.  The workgroup keeps h and c of the previous
// diagonal in LDS, indexed by row (rows without a pixel hold zeros, which is also what a
// predecessor outside the image contributes); a lane's entries of the recurrent matrices
// [R_u ; R_v] never change and stay in registers for the whole scan.
//
// Forward step: [16 rows x 2H] * [2H x 5H] on the matrix cores (v_mfma_f32_16x16x4_f32), one wavefront
// per (gate, 16 units): 16 MFMAs and one nonlinearity on four units per lane; the output-gate wavefronts
// collect the other activated gates from LDS and do the cell update.  The input part X W + b comes from
// a whole-image product, prefetched one diagonal ahead, or, for one input value per pixel, is formed
// in the kernel.
// Backward step (diagonals in reverse): d h = [d a(r+1) | d a(r)] of diagonal s+1 times
// [R_u ; R_v]^T, K = 10H, split five ways over the same wavefronts; the gate derivatives follow with one
// lane per (row, unit).  d a overwrites the gates in place; [h_up | h_left] of every pixel is kept from
// the forward pass so that d R_u and d R_v are one whole-image product each afterwards.
#include "rlstm_internal.h"
#include <algorithm>
#include <type_traits>

namespace rlstm {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kBand = 16;      // image rows a workgroup holds (whole 16-row MFMA tiles)
constexpr int kTiles = kBand / 16;
constexpr int kMaxBands = 256 / kBand;

// Gate functions on the hardware exponential (v_exp_f32, 1 ulp) and reciprocal (v_rcp_f32, 1 ulp): the
// gating of 8 (row, unit) pairs per lane is as long as the step's matrix product, so the libm expf
// (a dozen instructions more per call) would be a third of the step.  Absolute error ~2e-7.
__device__ __forceinline__ float md_exp(float u) { return __builtin_amdgcn_exp2f(u * 1.44269504088896341f); }
__device__ __forceinline__ float md_sigmoid(float u) { return __builtin_amdgcn_rcpf(1.0f + md_exp(-u)); }
__device__ __forceinline__ float md_tanh(float u) { return 2.0f * __builtin_amdgcn_rcpf(1.0f + md_exp(-2.0f * u)) - 1.0f; }

struct MdParams {
  float* zg[4];            // [P, 5H]: X W + b -> gates i|f_u|f_v|o|g -> d a
  float* c[4];             // [P, H]
  float* hc[4];            // [P, S]: h_up | h_left (| x) of every pixel, row stride S
  const float* Ru[4];      // [H, 5H]
  const float* Rv[4];
  float* y;                // forward: [P, 4H] output
  const float* dy;         // backward: [P, 4H]
  float* dbpart;           // backward: [4 B][NB][5H] bias gradient of every (direction, image, band)
  unsigned long long* halo;   // rows handed from a band to its neighbour: (value, diagonal + 1) words
  unsigned* err;           // raised when a bounded wait expired
  const int32_t* widths;   // [B]
  const float* x;          // forward with a one-value input (XIN): [P] pixels
  const float* W[4];       //   [1, 5H] input weights per direction
  const float* bias[4];    //   [5H]
  int Hh, Ww, B, H, S, NB;
  int mute_wg;             // test hook: this workgroup hands no row on (-1: none)
  unsigned long long wait_ticks;   // bound of a wait for a handed row, in ticks of the 100 MHz wall clock
};

// scan coordinates (row r, column q) of image n, direction (du, dv), image width wn -> pixel index
__device__ __forceinline__ size_t md_pixel(const MdParams& p, int du, int dv, int wn, int n, int r, int q) {
  const int u = du > 0 ? r : p.Hh - 1 - r;
  const int v = dv > 0 ? q : wn - 1 - q;
  return ((size_t)u * p.Ww + v) * p.B + n;
}

// four consecutive floats at q: one 16-byte access when the caller knows q is 16-byte aligned (VEC)
template <bool VEC>
__device__ __forceinline__ floatx4 ld4(const float* q, int nvalid) {
  if (VEC) return *reinterpret_cast<const floatx4*>(q);
  floatx4 v = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 4; ++i) if (i < nvalid) v[i] = q[i];
  return v;
}
template <bool VEC>
__device__ __forceinline__ void st4(float* q, floatx4 v, int nvalid) {
  if (VEC) { *reinterpret_cast<floatx4*>(q) = v; return; }
#pragma unroll
  for (int i = 0; i < 4; ++i) if (i < nvalid) q[i] = v[i];
}

// ---- rows handed between the bands of one scan -------------------------------------------------
// The image rows of a scan are cut into bands of kBand rows, one workgroup each.  A band needs, per
// anti-diagonal, one row of its neighbour (forward: h, c of the last row of the band above; backward:
// d a and f_u * d c~ of the first row of the band below).  The dependency runs one way, so the
// neighbour simply runs a diagonal or two ahead and nobody waits for a round trip.  Every value
// travels as one 64-bit word (value, diagonal + 1) written and read with device-scope accesses,
// so the reader polls the data itself; the words are cleared before every pass; waits are bounded.
constexpr unsigned long long kMdWaitTicks = 200000000ull;     // 2 s of the 100 MHz wall clock

__device__ __forceinline__ unsigned long long md_ld_word(const unsigned long long* q) {
  return __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void md_st_word(unsigned long long* q, float v, int diag) {
  __hip_atomic_store(q, ((unsigned long long)(unsigned)(diag + 1) << 32) | __float_as_uint(v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
// waits until word w (already loaded once) carries diagonal `diag`; false: gave up
__device__ __forceinline__ bool md_wait_word(const unsigned long long* q, unsigned long long& w, int diag, unsigned* err,
                                             unsigned long long ticks) {
  unsigned n = 0;
  unsigned long long t0 = 0;
  while ((unsigned)(w >> 32) != (unsigned)(diag + 1)) {
    w = md_ld_word(q);
    if ((++n & 255u) == 0) {
      const unsigned long long now = wall_clock64();
      if (t0 == 0) t0 = now;
      else if (now - t0 > ticks) return false;
      if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) return false;
    }
  }
  return true;
}

// VEC: H is a multiple of 4, so every group of four units starts 16-byte aligned in all tensors.
// Workgroup = (band of 16 rows, direction, image).
// Forward scan.  One wavefront per (gate, 16 units): 5 * HT wavefronts, one more that takes the rows handed from
// the band above and one that hands this band's last row to the band below (so that no gate wavefront, which the
// next step waits for, spends time on it).  A step's product
// a^T = [R_u ; R_v]^T [h_up | h_left]^T is then 16 MFMAs per wavefront instead of 80, and a lane applies one
// nonlinearity to its four units instead of five; the wavefronts of the output gate pick up the other four
// activated gates from LDS (same lane, one 16-byte read each) and do the cell update.  The lane's 16 matrix
// operands (its column of [R_u ; R_v] for its gate and unit) never change and stay in registers.
// XIN: the input has one value per pixel (grayscale images): the input part b + x W of the pre-activation is formed
// here from x and this lane's weights and biases instead of being read from zg, and x is written next to
// [h_up | h_left] for the weight-gradient product.
// The gate wavefronts store (gates, c, y, [h_up | h_left]) and therefore never load inside the loop: a wavefront's
// memory counter retires in order, so waiting for a load would mean waiting for the stores issued before it.
template <int HT, bool VEC, int XM>
__global__ __launch_bounds__(64 * (5 * HT + 2)) void mdlstm_fwd_kernel(MdParams p) {
  constexpr bool XIN = XM != 0;        // XM: 0 input part read from zg, 1 x read from HBM, 2 the band's x staged in LDS
  static_assert(kTiles == 1, "one 16-row tile per band");
  constexpr int NTH = 64 * (5 * HT + 2);   // two more wavefronts: one takes the rows handed from the band above, one hands this band's last row on
  constexpr int HP = 16 * HT;          // padded units
  constexpr int KS = 2 * HP / 4;       // MFMA k-steps
  constexpr int LDH = HP + 1;
  constexpr int HW = 2 * HP;           // words of a handed row: h | c
  extern __shared__ __align__(16) float lds[];
  float* hb = lds;                                   // [2][kBand + 1][LDH]; entry 0 is the row above the band
  float* cb = hb + 2 * (kBand + 1) * LDH;            // same for c
  floatx4* gact = reinterpret_cast<floatx4*>(cb + 2 * (kBand + 1) * LDH);   // [i, f_u, f_v, g][HT][64 lanes]
  int* gaveup = reinterpret_cast<int*>(gact + 4 * HT * 64);                  // raised when a bounded wait expired (16 bytes)
  float* xs = reinterpret_cast<float*>(gaveup + 4);                          // XIN, staged: [kBand][Ww] x in scan coordinates

  const int dn = blockIdx.x % (4 * p.B), band = blockIdx.x / (4 * p.B);   // bands above come first in the grid
  const int d = dn & 3, n = dn >> 2;
  const int du = (d & 2) ? -1 : 1, dv = (d & 1) ? -1 : 1;
  const int H = p.H, Hh = p.Hh;
  const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Wavefront 5 HT only moves the handed rows in: it issues the only global loads of the scan.  A wavefront's memory
  // counter retires in order, so a wavefront that waits for a load waits for every store it issued before, and
  // a store to HBM takes about as long as a step; the gate wavefronts, which store, therefore never load.
  const bool is_halo = wave == 5 * HT, is_sender = wave == 5 * HT + 1;
  const int g = (is_halo || is_sender) ? 5 : wave / HT, ht = wave % HT;     // gate (i, f_u, f_v, o, g) and group of 16 units of this wavefront
  const int lr = l16;                          // row inside the band
  const int r = kBand * band + lr;             // row of this lane
  const int jm = 16 * ht + l16;                // unit whose column this lane feeds to the MFMA (A operand row)
  const int j0 = 16 * ht + 4 * lq;             // first of the four units this lane holds (accumulator rows)
  const int nv = (is_halo || is_sender) ? 0 : min(max(H - j0, 0), 4);       // how many of them exist
  const int wn = min(max(p.widths[n], 0), p.Ww);
  const int rows_here = min(Hh - kBand * band, kBand);
  const int slot = g < 3 ? g : 3;              // where this gate's activations go in gact (the output gate has none)
  const float act_scale = g == 4 ? 2.f : 1.f, act_shift = 1.f - act_scale;

  // A[m][k] = [R_u ; R_v][k][gate column of unit m]
  float ra[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int k = 4 * ks + lq, kk = k % HP;
    const float* R = k < HP ? p.Ru[d] : p.Rv[d];
    ra[ks] = (!is_halo && !is_sender && kk < H && jm < H) ? R[(size_t)kk * 5 * H + g * H + jm] : 0.f;
  }
  for (int idx = tid; idx < 2 * (kBand + 1) * LDH; idx += NTH) { hb[idx] = 0.f; cb[idx] = 0.f; }
  if (tid == 0) *gaveup = 0;
  // One input value per pixel: the band's x goes to LDS once, so that no step of the scan waits for a load from
  // HBM (the memory counter retires in order: waiting for a load issued after a step's stores means waiting for
  // the stores, about as long as a step; issuing the load first was measured slower still).
  constexpr bool xstaged = XM == 2;
  if (xstaged) {
    for (int idx = tid; idx < rows_here * wn; idx += NTH) {
      const int rr = idx / wn, qq = idx % wn;
      xs[rr * p.Ww + qq] = p.x[md_pixel(p, du, dv, wn, n, kBand * band + rr, qq)];
    }
  }
  __syncthreads();

  float* zgd = p.zg[d];
  float* cd = p.c[d];
  float* hcd = p.hc[d];
  // diagonals on which this band has pixels
  const int s_lo = kBand * band, s_hi = wn > 0 ? kBand * band + rows_here - 1 + wn - 1 : s_lo - 1;
  const int ndiag = Hh + p.Ww;
  // the row above the band (last row of the band above) has pixels on diagonals s_lo - 1 .. s_lo - 1 + wn - 1
  const bool takes = band > 0, gives = band < p.NB - 1 && (int)blockIdx.x != p.mute_wg;
  const unsigned long long* halo_in = takes ? p.halo + ((size_t)dn * (p.NB - 1) + (band - 1)) * ndiag * 64 : p.halo;
  unsigned long long* halo_out = gives ? p.halo + ((size_t)dn * (p.NB - 1) + band) * ndiag * 64 : p.halo;
  const bool hands = is_halo && lane < HW;     // the lanes that move the handed row in
  const bool sends = is_sender && lane < HW;   // the lanes that hand this band's last row on (a wavefront that never loads)

  // h, c of the row above on diagonal sd -> entry 0 of the given buffers; returns false when a wait expired
  unsigned long long hw = 0;
  auto halo_issue = [&](int sd) {
    if (hands && takes && sd >= s_lo - 1 && sd <= s_lo - 1 + wn - 1) hw = md_ld_word(halo_in + (size_t)sd * 64 + lane);
  };
  auto halo_take = [&](int sd, float* hdst, float* cdst) -> bool {
    if (!hands) return true;
    float v = 0.f;
    bool good = true;
    if (takes && sd >= s_lo - 1 && sd <= s_lo - 1 + wn - 1) {
      good = md_wait_word(halo_in + (size_t)sd * 64 + lane, hw, sd, p.err, p.wait_ticks);
      v = __uint_as_float((unsigned)hw);
    }
    if (lane < HP) hdst[lane] = v; else cdst[lane - HP] = v;
    return good;
  };

  // input part of this lane's gate, row and four units on diagonal s
  floatx4 zr = floatx4{0.f, 0.f, 0.f, 0.f};
  floatx4 wx = zr, bx = zr;            // XIN: weights and biases of this lane's four units for its gate
  float xcur = 0.f;                    // XIN: x of the pixel of the diagonal at hand
  if (XIN) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      wx[i] = i < nv ? p.W[d][g * H + j0 + i] : 0.f;
      bx[i] = i < nv ? p.bias[d][g * H + j0 + i] : 0.f;
    }
  }
  auto prefetch = [&](int s) {
    const int q = s - r;
    const bool ok = lr < rows_here && q >= 0 && q < wn && s <= s_hi && nv > 0;
    const size_t pix = ok ? md_pixel(p, du, dv, wn, n, r, q) : 0;
    if (XIN) xcur = ok ? (xstaged ? xs[lr * p.Ww + q] : p.x[pix]) : 0.f;   // used after the step's MFMAs
    else zr = ok ? ld4<VEC>(zgd + pix * 5 * H + g * H + j0, nv) : floatx4{0.f, 0.f, 0.f, 0.f};
  };
  prefetch(s_lo);
  int fail = 0;
  {
    // the row above on the diagonal before the first one
    float* hprev0 = hb + ((s_lo + 1) & 1) * (kBand + 1) * LDH;
    float* cprev0 = cb + ((s_lo + 1) & 1) * (kBand + 1) * LDH;
    halo_issue(s_lo - 1);
    if (!halo_take(s_lo - 1, hprev0, cprev0)) fail = 1;
  }
  if (fail) *gaveup = 1;
  __syncthreads();
  if (*gaveup) {
    if (tid == 0) __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return;
  }

  // The wavefront that takes the handed rows runs a loop of its own with the same barriers, so that the gate
  // wavefronts' loop holds no load and hence no wait on the memory counter.
  if (is_halo) {
    for (int s = s_lo; s <= s_hi; ++s) {
      halo_issue(s);                   // has the whole step to arrive
      __syncthreads();
      // the row above on this diagonal, for the next step (entry 0 of the buffers nobody reads in this step)
      if (!halo_take(s, hb + (s & 1) * (kBand + 1) * LDH, cb + (s & 1) * (kBand + 1) * LDH)) *gaveup = 1;
      __syncthreads();
      if (*gaveup) return;
    }
  } else if (is_sender) {
    for (int s = s_lo; s <= s_hi; ++s) {
      __syncthreads();
      __syncthreads();
      if (*gaveup) return;
      if (gives && sends) {            // last row of the band to the band below
        const float* hcur = hb + (s & 1) * (kBand + 1) * LDH;
        const float* ccur = cb + (s & 1) * (kBand + 1) * LDH;
        md_st_word(halo_out + (size_t)s * 64 + lane, lane < HP ? hcur[kBand * LDH + lane] : ccur[kBand * LDH + lane - HP], s);
      }
    }
  } else
  for (int s = s_lo; s <= s_hi; ++s) {
    const float* hprev = hb + ((s + 1) & 1) * (kBand + 1) * LDH;
    const float* cprev = cb + ((s + 1) & 1) * (kBand + 1) * LDH;
    float* hcur = hb + (s & 1) * (kBand + 1) * LDH;
    float* ccur = cb + (s & 1) * (kBand + 1) * LDH;

    // accumulator rows: units j0 .. j0+3 of this gate; column: the image row of this lane.
    // B[k][n]: k < HP: h of the row above (entry index = row), else h of the same row (entry index row + 1)
    floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = acc0;
    const float* brow = hprev + lr * LDH;
    // all of the step's B operands are fetched before the first MFMA (left to itself the compiler reuses two
    // registers and waits for an LDS read in front of every pair of MFMAs)
    float hv[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k = 4 * ks + lq;
      hv[ks] = k < HP ? brow[k] : brow[LDH + k - HP];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < KS; ks += 2) {
      acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[ks], hv[ks], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[ks + 1], hv[ks + 1], acc1, 0, 0, 0);
    }

    const int q = s - r;
    const bool ok = lr < rows_here && q >= 0 && q < wn && nv > 0;
    const size_t pix = ok ? md_pixel(p, du, dv, wn, n, r, q) : 0;
    if (XIN) zr = bx + xcur * wx;
    // sigmoid for the four gates, tanh(a) = 2 sigmoid(2a) - 1 for the cell input: one branch-free form
    floatx4 act;
#pragma unroll
    for (int i = 0; i < 4; ++i) act[i] = act_scale * md_sigmoid(act_scale * (acc0[i] + acc1[i] + zr[i])) + act_shift;
    if (g != 3) gact[(slot * HT + ht) * 64 + lane] = act;
    __syncthreads();

    floatx4 ct = floatx4{0.f, 0.f, 0.f, 0.f}, hn = ct, h_up = ct, h_left = ct;
    if (g == 3) {
      const floatx4 gi = gact[(0 * HT + ht) * 64 + lane], gfu = gact[(1 * HT + ht) * 64 + lane];
      const floatx4 gfv = gact[(2 * HT + ht) * 64 + lane], gg = gact[(3 * HT + ht) * 64 + lane];
      // every LDS read of the update comes before its first LDS write (the compiler cannot tell that the rows it
      // writes are not the rows it reads, and would wait after every unit)
      floatx4 c_up, c_left;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = j0 + i;
        h_up[i] = hprev[lr * LDH + j]; h_left[i] = hprev[(lr + 1) * LDH + j];
        c_up[i] = cprev[lr * LDH + j]; c_left[i] = cprev[(lr + 1) * LDH + j];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ct[i] = gfu[i] * c_up[i] + gfv[i] * c_left[i] + gi[i] * gg[i];
        hn[i] = act[i] * md_tanh(ct[i]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool oki = ok && i < nv;
        hcur[(lr + 1) * LDH + j0 + i] = oki ? hn[i] : 0.f;
        ccur[(lr + 1) * LDH + j0 + i] = oki ? ct[i] : 0.f;
      }
    }
    // the next diagonal only needs the LDS rows: the stores to HBM and the next prefetch follow the barrier
    __syncthreads();
    if (*gaveup) {
      if (tid == 0) __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return;
    }
    if (ok) {
      st4<VEC>(zgd + pix * 5 * H + g * H + j0, act, nv);
      if (g == 3) {
        st4<VEC>(cd + pix * H + j0, ct, nv);
        st4<VEC>(p.y + pix * 4 * H + d * H + j0, hn, nv);
        st4<VEC>(hcd + pix * p.S + j0, h_up, nv);
        st4<VEC>(hcd + pix * p.S + H + j0, h_left, nv);
        if (XIN && j0 == 0) hcd[pix * p.S + 2 * H] = xcur;
      }
    }
    prefetch(s + 1);
  }

  // pixels beyond the image's width: y = 0, and zeros where the products after the backward pass read
  const int npad = (p.Ww - wn) * rows_here;
  for (int idx = tid; idx < npad * H; idx += NTH) {
    const int jj = idx % H, cell = idx / H;
    const int rr = kBand * band + cell / (p.Ww - wn), v = wn + cell % (p.Ww - wn);
    const int u = du > 0 ? rr : Hh - 1 - rr;
    const size_t pix = ((size_t)u * p.Ww + v) * p.B + n;
    p.y[pix * 4 * H + d * H + jj] = 0.f;
    cd[pix * H + jj] = 0.f;
    hcd[pix * p.S + jj] = 0.f;
    hcd[pix * p.S + H + jj] = 0.f;
    if (XIN && jj == 0) hcd[pix * p.S + 2 * H] = 0.f;
  }
}


// Backward scan.  d h^T of a diagonal = [R_u ; R_v] [d a(row + 1) | d a(row)]^T of the diagonal done before it, a
// contraction over K = 10 HP.  A step has two phases with a barrier between them.
// Product: 5 * HT compute wavefronts; wavefront (g, ht) takes the columns of gate g (a fifth of K) for the 16 units
// of ht (16 MFMAs for HT = 2, its operands of [R_u ; R_v] in registers) and leaves its partial sums in LDS.
// Gate derivatives: one lane per (row, unit) of the diagonal (16 * HP lanes, HP / 4 of the compute wavefronts): it
// adds the five partial sums in a fixed order and forms the five d a of its pixel and unit.  What limits a step is
// the number of vector instructions the workgroup issues (a SIMD issues one wavefront instruction per 4 cycles, and
// the wavefronts of a SIMD share it), so every value is computed exactly once and the lane's addresses advance by a
// constant per diagonal instead of being recomputed.
// A wavefront's memory counter retires in order, so a wavefront that waits for a load waits for every store it issued
// before; loads and stores are therefore kept in different wavefronts: the compute wavefronts only load (two diagonals
// ahead, see below), two more wavefronts only store (d a rows out of LDS, and the row handed to the band above) and
// one only takes the row handed from the band below.
template <int HT, bool VEC>
__global__ __launch_bounds__(64 * (5 * HT + 3)) void mdlstm_bwd_kernel(MdParams p) {
  static_assert(kTiles == 1, "one 16-row tile per band");
  constexpr int NC = 5 * HT;           // compute wavefronts
  constexpr int NTH = 64 * (NC + 3);
  constexpr int HP = 16 * HT;
  constexpr int NG = 5 * HP;
  constexpr int KS = 2 * HP / 4;       // MFMA k-steps of one wavefront: a fifth of K = 2 NG
  constexpr int LDZ = NG + 4;          // LDS row stride of the d a rows (a multiple of 4: rows stay 16-byte aligned)
  constexpr int LDH = HP + 1;
  constexpr int HW = NG + HP;          // words of a handed row: d a | f_u * d c~
  extern __shared__ __align__(16) float lds[];
  constexpr int LDP = HP + 4;          // row stride of the partial sums (a multiple of 4)
  float* part = lds;                                 // [5][16 rows][LDP]: partial d h of every fifth of K
  float* dzb = lds + 5 * 16 * LDP;                   // [kBand + 1][LDZ]: d a of the diagonal done last; entry kBand is the row below the band
  float* dcu = dzb + (kBand + 1) * LDZ;              // [2][kBand + 1][LDH]: f_u * d c~ of a diagonal's pixels; entry kBand: row below
  float* dcv = dcu + 2 * (kBand + 1) * LDH;          // same with f_v
  int* gaveup = reinterpret_cast<int*>(dcv + 2 * (kBand + 1) * LDH);   // raised when a bounded wait expired

  // Workgroups beyond the scan's own (they land on the CUs the scan leaves idle, and come last in the grid) clear
  // d a of the pixel slots beyond the images' widths, which the products over all pixel slots read.
  const int nscan = 4 * p.B * p.NB;
  if ((int)blockIdx.x >= nscan) {
    const int cols = 5 * p.H;
    for (int pair = (int)blockIdx.x - nscan; pair < p.Hh * p.B; pair += (int)gridDim.x - nscan) {
      const int nn = pair % p.B, u = pair / p.B;
      const int wn = min(max(p.widths[nn], 0), p.Ww);
      const int total = (p.Ww - wn) * cols;
      for (int idx = threadIdx.x; idx < total; idx += NTH) {
        const int v = wn + idx / cols, col = idx % cols;
        const size_t o = (((size_t)u * p.Ww + v) * p.B + nn) * cols + col;
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) p.zg[dd][o] = 0.f;
      }
    }
    return;
  }
  // bands below come first in the grid
  const int dn = blockIdx.x % (4 * p.B), band = p.NB - 1 - blockIdx.x / (4 * p.B);
  const int d = dn & 3, n = dn >> 2;
  const int du = (d & 2) ? -1 : 1, dv = (d & 1) ? -1 : 1;
  const int H = p.H, Hh = p.Hh;
  const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool computes = wave < NC, stores = wave == NC || wave == NC + 1, is_halo = wave == NC + 2;
  const int g = computes ? wave / HT : 0, ht = wave % HT;   // gate, which is also the fifth of K, and group of 16 units
  const int lr = l16;                          // row inside the band
  const int jm = 16 * ht + l16;                // unit whose row of [R_u ; R_v] this lane feeds to the MFMA
  const int j0 = 16 * ht + 4 * lq;             // first of the four units this lane handles
  const int wn = min(max(p.widths[n], 0), p.Ww);
  const int rows_here = min(Hh - kBand * band, kBand);

  // The fifth of K of wavefront (g, ht): the columns of gate g, first of R_u (against d a of the row below,
  // row + 1), then of R_v (against d a of the same row).  A[m][k] = R[unit m][column k of gate g].
  float ra[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int jj = 4 * (ks % (KS / 2)) + lq;
    const float* R = ks < KS / 2 ? p.Ru[d] : p.Rv[d];
    ra[ks] = (computes && jj < H && jm < H) ? R[(size_t)jm * 5 * H + g * H + jj] : 0.f;
  }
  const float* bbase = dzb + lr * LDZ + g * HP + lq;   // B[k][row]: + LDZ + 4 ks for the first half, + 4 (ks - KS/2) for the second
  for (int idx = tid; idx < (kBand + 1) * LDZ; idx += NTH) dzb[idx] = 0.f;
  for (int idx = tid; idx < 2 * (kBand + 1) * LDH; idx += NTH) { dcu[idx] = 0.f; dcv[idx] = 0.f; }
  if (tid == 0) *gaveup = 0;
  __syncthreads();

  float* zgd = p.zg[d];
  const float* cd = p.c[d];
  const int s_lo = kBand * band, s_hi = wn > 0 ? kBand * band + rows_here - 1 + wn - 1 : s_lo - 1;
  const int ndiag = Hh + p.Ww;
  // the row below the band (first row of the band below) has pixels on diagonals b_lo .. b_lo + wn - 1
  const int b_lo = kBand * (band + 1);
  const bool takes = band < p.NB - 1, gives = band > 0 && (int)blockIdx.x != p.mute_wg;
  const unsigned long long* halo_in = takes ? p.halo + ((size_t)dn * (p.NB - 1) + band) * ndiag * 192 : p.halo;
  unsigned long long* halo_out = gives ? p.halo + ((size_t)dn * (p.NB - 1) + (band - 1)) * ndiag * 192 : p.halo;

  // d a and f_u * d c~ of the row below on diagonal sd -> entry kBand of dzb / of dcu's buffer for sd
  unsigned long long hw[3] = {0, 0, 0};
  auto halo_issue = [&](int sd) {
    if (takes && sd >= b_lo && sd <= b_lo + wn - 1)
#pragma unroll
      for (int k = 0; k < 3; ++k)
        if (lane + 64 * k < HW) hw[k] = md_ld_word(halo_in + (size_t)sd * 192 + lane + 64 * k);
  };
  auto halo_take = [&](int sd) -> bool {
    bool good = true;
    const bool have = takes && sd >= b_lo && sd <= b_lo + wn - 1;
    float* dcu_dst = dcu + (sd & 1) * (kBand + 1) * LDH;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int w = lane + 64 * k;
      if (w >= HW) continue;
      float v = 0.f;
      if (have) {
        good = md_wait_word(halo_in + (size_t)sd * 192 + w, hw[k], sd, p.err, p.wait_ticks) && good;
        v = __uint_as_float((unsigned)hw[k]);
      }
      if (w < NG) dzb[kBand * LDZ + w] = v; else dcu_dst[kBand * LDH + w - NG] = v;
    }
    return good;
  };

  // The wavefront whose wait expired raises the flag in HBM itself: a store in the compute wavefronts' loop, even on
  // a path that leaves it, would make the compiler wait for every load in flight on each diagonal (loads and
  // stores pending on one counter count as unordered).
  auto give_up = [&]() {
    *gaveup = 1;
    __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
  if (is_halo) {
    // the row below on the diagonal after the last one
    halo_issue(s_hi + 1);
    if (!halo_take(s_hi + 1)) give_up();
  }
  __syncthreads();
  if (*gaveup) return;

  // Every wavefront passes the same two barriers per diagonal: A after the partial products (the d a rows of the
  // diagonal before have been read), B when the LDS rows of the diagonal are complete.
  if (is_halo) {
    for (int s = s_hi; s >= s_lo; --s) {
      if (s > s_lo) halo_issue(s);     // has the whole step to arrive
      __syncthreads();
      const int stop = *gaveup;        // raised during the diagonal before: every wavefront reads it here
      if (s > s_lo && !halo_take(s)) give_up();
      __syncthreads();
      if (stop) return;
    }
    __syncthreads();                   // the barrier of the bias-gradient sum below
    return;
  }

  if (stores) {
    // lane -> (row, eight lanes a row); the row's d a leave LDS 16 bytes at a time
    const int t = 64 * (wave - NC) + lane, row = t >> 3, c8 = t & 7;
    auto store_rows = [&](int s) {
      if (gives && wave == NC) {       // first row of the band to the band above, first: that band waits for it
        const float* dcu_s = dcu + (s & 1) * (kBand + 1) * LDH;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
          const int w = lane + 64 * k;
          if (w < HW) md_st_word(halo_out + (size_t)s * 192 + w, w < NG ? dzb[w] : dcu_s[w - NG], s);
        }
      }
      const int q = s - (kBand * band + row);
      if (row < rows_here && q >= 0 && q < wn) {
        float* zrow = zgd + md_pixel(p, du, dv, wn, n, kBand * band + row, q) * 5 * H;
#pragma unroll
        for (int k = 0; k < (NG / 4 + 7) / 8; ++k) {
          const int colf = 4 * (c8 + 8 * k), gk = colf / HP, jj = colf % HP;
          if (colf < NG && jj < H) st4<VEC>(zrow + gk * H + jj, *reinterpret_cast<const floatx4*>(dzb + row * LDZ + colf), min(H - jj, 4));
        }
      }
    };
    for (int s = s_hi; s >= s_lo; --s) {
      if (s < s_hi) store_rows(s + 1);
      __syncthreads();
      const int stop = *gaveup;
      __syncthreads();
      if (stop) return;
    }
    if (s_hi >= s_lo) store_rows(s_lo);
    __syncthreads();                   // the barrier of the bias-gradient sum below
    return;
  }

  // ---- compute wavefronts ----
  floatx4* part_w = reinterpret_cast<floatx4*>(part + (g * 16 + lr) * LDP + j0);   // where the product phase leaves its sums

  // gate-derivative phase: lane -> (row, unit) of the band
  constexpr int NE = HP / 4;           // wavefronts that take part in it
  const bool elem = wave < NE;
  const int er = (64 * wave + lane) / HP, ej = (64 * wave + lane) % HP;   // row inside the band, unit
  const int rr = kBand * band + er;    // row of this lane's pixels
  const bool live = elem && er < rows_here && ej < H;
  // element offsets of the lane's pixel on diagonal s in the tensors with 5H, H and 4H values per pixel; they move
  // by a constant from one diagonal to the next (q falls by one: the pixel index moves by -dv * B), also while the
  // lane has no pixel on the diagonal, when nothing is loaded
  long long oz, oc, oy;
  {
    const long long u = du > 0 ? rr : Hh - 1 - rr;
    const long long q0 = (long long)s_hi - rr, v0 = dv > 0 ? q0 : wn - 1 - q0;
    const long long pix = (u * p.Ww + v0) * p.B + n;
    oz = pix * 5 * H + ej; oc = pix * H + ej; oy = pix * 4 * H + d * H + ej;
  }
  const long long pstep = -(long long)dv * p.B;                                     // pixel index, per diagonal
  const long long c_up = -(long long)du * p.Ww * p.B * H, c_left = -(long long)dv * p.B * H;   // c of the predecessors, relative to oc
  const float* dyd = p.dy;
  // Two register sets, loaded two diagonals ahead.  Every load is issued on every diagonal (a lane without a pixel
  // there reads the tensors' first words and drops them when it uses them): with no branch around the loads the
  // wait for one set leaves the other, younger one in flight.
  struct In { float gi, gfu, gfv, go, gg, cc, cu, cl, dy; };
  auto issue = [&](In& in, int s) {
    const int q = s - rr;
    const bool ok = live && s >= s_lo && q >= 0 && q < wn;
    const long long az = ok ? oz : 0, ac = ok ? oc : 0, ay = ok ? oy : 0;
    const long long au = (ok && rr >= 1) ? oc + c_up : 0, al = (ok && q >= 1) ? oc + c_left : 0;
    const float* z = zgd + az;
    in.cc = cd[ac];
    in.dy = dyd[ay];
    in.go = z[3 * H];
    in.gi = z[0]; in.gfu = z[H]; in.gfv = z[2 * H]; in.gg = z[4 * H];
    in.cu = cd[au];
    in.cl = cd[al];
    oz += pstep * 5 * H; oc += pstep * H; oy += pstep * 4 * H;
  };

  float dbacc[5] = {0.f, 0.f, 0.f, 0.f, 0.f};   // bias gradient of the lane's unit over its row's pixels
  // one diagonal; false: a wait expired somewhere in the workgroup
  auto step = [&](auto takes_part, In& in, int s) -> bool {
    constexpr bool ELEM = decltype(takes_part)::value;
    const float* dcu_prev = dcu + ((s + 1) & 1) * (kBand + 1) * LDH;
    const float* dcv_prev = dcv + ((s + 1) & 1) * (kBand + 1) * LDH;
    float* dcu_cur = dcu + (s & 1) * (kBand + 1) * LDH;
    float* dcv_cur = dcv + (s & 1) * (kBand + 1) * LDH;
    // all of the step's B operands are fetched before the first MFMA; two accumulators so that consecutive MFMAs
    // do not wait for each other
    float hv[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) hv[ks] = ks < KS / 2 ? bbase[LDZ + 4 * ks] : bbase[4 * (ks - KS / 2)];
    __builtin_amdgcn_sched_barrier(0);
    floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = acc0;
#pragma unroll
    for (int ks = 0; ks < KS; ks += 2) {
      acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[ks], hv[ks], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[ks + 1], hv[ks + 1], acc1, 0, 0, 0);
    }
    *part_w = acc0 + acc1;
    __syncthreads();     // A

    // a flag raised during the diagonal before is seen here by every wavefront alike
    const int stop = *gaveup;
    if (ELEM) {
      const int q = s - rr;
      const bool ok = live && q >= 0 && q < wn;
      const float* pr = part + er * LDP + ej;
      const float p0 = pr[0], p1 = pr[16 * LDP], p2 = pr[2 * 16 * LDP], p3 = pr[3 * 16 * LDP], p4 = pr[4 * 16 * LDP];
      const float su = dcu_prev[(er + 1) * LDH + ej], sv = dcv_prev[er * LDH + ej];
      const float gi = in.gi, gfu = in.gfu, gfv = in.gfv, go = in.go, gg = in.gg;
      const float cu = rr >= 1 ? in.cu : 0.f, cl = q >= 1 ? in.cl : 0.f;   // c of a predecessor outside the image is zero
      const float tc = md_tanh(in.cc);
      const float dh = in.dy + ((((p0 + p1) + p2) + p3) + p4);
      const float dct = su + sv + dh * go * (1.0f - tc * tc);
      const float dz0 = ok ? dct * gg * gi * (1.0f - gi) : 0.f;
      const float dz1 = ok ? dct * cu * gfu * (1.0f - gfu) : 0.f;
      const float dz2 = ok ? dct * cl * gfv * (1.0f - gfv) : 0.f;
      const float dz3 = ok ? dh * tc * go * (1.0f - go) : 0.f;
      const float dz4 = ok ? dct * gi * (1.0f - gg * gg) : 0.f;
      float* zr = dzb + er * LDZ + ej;
      zr[0] = dz0; zr[HP] = dz1; zr[2 * HP] = dz2; zr[3 * HP] = dz3; zr[4 * HP] = dz4;
      dcu_cur[er * LDH + ej] = ok ? dct * gfu : 0.f;
      dcv_cur[er * LDH + ej] = ok ? dct * gfv : 0.f;
      dbacc[0] += dz0; dbacc[1] += dz1; dbacc[2] += dz2; dbacc[3] += dz3; dbacc[4] += dz4;
      issue(in, s - 2);
    }
    __syncthreads();     // B
    return stop == 0;
  };

  // nothing older than the two register sets may be in flight when the loop starts, or the waits inside it turn
  // into waits for everything (vmcnt(0), expcnt and lgkmcnt left alone)
  __builtin_amdgcn_s_waitcnt(0x0F70);
  // The wavefronts without a part in the gate derivatives run a loop of their own: a branch around the loads inside
  // one common loop would again make every wait a wait for everything.
  In inA, inB;
  if (elem) {
    issue(inA, s_hi);
    issue(inB, s_hi - 1);
    for (int s = s_hi; s >= s_lo; s -= 2) {
      if (!step(std::true_type{}, inA, s)) return;
      if (s - 1 < s_lo) break;
      if (!step(std::true_type{}, inB, s - 1)) return;
    }
  } else {
    for (int s = s_hi; s >= s_lo; --s)
      if (!step(std::false_type{}, inA, s)) return;
  }

  // bias gradient of this (direction, image, band): the 16 rows of a unit are added in row order
  float* stage = part;                               // [5 HP][16 rows]; the last step's partial sums have been read
  if (elem) {
#pragma unroll
    for (int k = 0; k < 5; ++k) stage[(k * HP + ej) * 16 + er] = dbacc[k];
  }
  __syncthreads();
  for (int idx = tid; idx < 5 * HP; idx += 64 * NC) {
    const int gk = idx / HP, jo = idx % HP;
    if (jo < H) {
      float sum = 0.f;
      for (int l = 0; l < 16; ++l) sum += stage[idx * 16 + l];
      p.dbpart[((size_t)dn * p.NB + band) * 5 * H + gk * H + jo] = sum;
    }
  }
}

// db[d][col] = sum over the images and their bands, in that order
struct MdDbParams { float* db[4]; const float* dbpart; int B, NB, n; };
__global__ __launch_bounds__(64) void mdlstm_db_sum_kernel(MdDbParams p) {
  const int i = blockIdx.x * 64 + threadIdx.x, d = blockIdx.y;
  if (i >= p.n) return;
  float sum = 0.f;
  for (int b = 0; b < p.B; ++b)
    for (int k = 0; k < p.NB; ++k) sum += p.dbpart[((size_t)(b * 4 + d) * p.NB + k) * p.n + i];
  p.db[d][i] = sum;
}

// clears the handed-row words before a pass; the forward pass (err != null) also clears the timeout flag, the
// backward pass leaves it: a timeout of the forward pass stays visible after the backward call
__global__ __launch_bounds__(256) void mdlstm_clear_kernel(unsigned long long* words, size_t n, unsigned* err) {
  const size_t gsz = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += gsz) words[i] = 0ull;
  if (err && blockIdx.x == 0 && threadIdx.x == 0) *err = 0u;
}

// x [P, D] into columns [2H, 2H + D) of the four [P, S] predecessor-output arrays, so that
// [h_up | h_left | x]^T dA gives dR_u, dR_v and dW in one product
struct MdXCopyParams { float* hc[4]; const float* x; size_t P; int D, H, S; };
__global__ __launch_bounds__(256) void mdlstm_xcopy_kernel(MdXCopyParams p) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= p.P * p.D) return;
  const size_t pix = idx / p.D;
  const int i = (int)(idx % p.D);
  const float v = p.x[idx];
#pragma unroll
  for (int d = 0; d < 4; ++d) p.hc[d][pix * p.S + 2 * p.H + i] = v;
}
// rows of the stacked gradient [2H + D, 5H] of every direction to the caller's dR_u, dR_v, dW
struct MdScatterParams { const float* stacked[4]; float* dRu[4]; float* dRv[4]; float* dW[4]; int D, H; };
__global__ __launch_bounds__(256) void mdlstm_scatter_kernel(MdScatterParams p) {
  const int n5 = 5 * p.H, rows = 2 * p.H + p.D;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * n5) return;
  const int row = idx / n5, col = idx % n5;
  for (int d = 0; d < 4; ++d) {
    const float v = p.stacked[d][idx];
    if (row < p.H) p.dRu[d][row * n5 + col] = v;
    else if (row < 2 * p.H) p.dRv[d][(row - p.H) * n5 + col] = v;
    else p.dW[d][(row - 2 * p.H) * n5 + col] = v;
  }
}

size_t md_lds_fwd(int HT) {
  const int HP = 16 * HT;
  return (size_t)4 * (kBand + 1) * (HP + 1) * sizeof(float) + (size_t)4 * HT * 64 * 16 + 16;
}
// room for a band's x values behind that, when it fits
size_t md_lds_xstage(int Ww) { return (size_t)kBand * Ww * sizeof(float); }
size_t md_lds_bwd(int HT) {
  const int HP = 16 * HT, NG = 5 * HP;
  return ((size_t)5 * 16 * (HP + 4) + (size_t)(kBand + 1) * (NG + 4) + (size_t)4 * (kBand + 1) * (HP + 1)) * sizeof(float) + 16;
}

template <typename K>
hipError_t md_launch(K kernel, int grid, int block, size_t lds, hipStream_t stream, MdParams& p) {
  const void* fn = reinterpret_cast<const void*>(kernel);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  void* args[] = {&p};
  return hipLaunchKernel(fn, dim3((unsigned)grid), dim3((unsigned)block), args, lds, stream);
}

int g_md_mute_wg = -1;
unsigned long long g_md_wait_ticks = 0;

MdParams md_params(const MdShape& s, const MdDir* dirs, const int32_t* widths) {
  MdParams p{};
  for (int d = 0; d < 4; ++d) {
    p.zg[d] = dirs[d].zg; p.c[d] = dirs[d].c; p.hc[d] = dirs[d].hc; p.Ru[d] = dirs[d].Ru; p.Rv[d] = dirs[d].Rv;
  }
  p.widths = widths; p.Hh = s.Hh; p.Ww = s.Ww; p.B = s.B; p.H = s.H; p.S = s.S;
  p.NB = (s.Hh + kBand - 1) / kBand;
  p.mute_wg = g_md_mute_wg;
  p.wait_ticks = g_md_wait_ticks ? g_md_wait_ticks : kMdWaitTicks;
  return p;
}

}  // namespace

namespace {
inline bool md_aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }
// groups of four units can be moved as one 16-byte access
bool md_vec(const MdShape& s, const MdDir* dirs, const float* yy) {
  bool v = s.H % 4 == 0 && md_aligned16(yy);
  for (int d = 0; d < 4; ++d) v = v && md_aligned16(dirs[d].zg) && md_aligned16(dirs[d].c) && md_aligned16(dirs[d].hc);
  return v;
}
}  // namespace

void mdlstm_test_hook(int mute_workgroup, unsigned long long wait_ticks) {
  g_md_mute_wg = mute_workgroup;
  g_md_wait_ticks = wait_ticks;
}

bool mdlstm_supported(const MdShape& s) { return s.Hh >= 1 && s.Hh <= kBand * kMaxBands && s.H >= 1 && s.H <= 32; }

// 64-bit words for the rows handed between bands (the backward pass needs the larger array)
size_t mdlstm_halo_words(const MdShape& s) {
  const size_t nb = (size_t)(s.Hh + kBand - 1) / kBand;
  return (size_t)4 * s.B * (nb - 1) * ((size_t)s.Hh + s.Ww) * 192;
}

namespace {
hipError_t md_clear(hipStream_t stream, const MdShape& s, unsigned long long* halo, unsigned* err, int words_per_diag) {
  const size_t nb = (size_t)(s.Hh + kBand - 1) / kBand;
  const size_t n = (size_t)4 * s.B * (nb - 1) * ((size_t)s.Hh + s.Ww) * words_per_diag;
  hipLaunchKernelGGL(mdlstm_clear_kernel, dim3(256), dim3(256), 0, stream, halo, n, err);
  return hipGetLastError();
}
}  // namespace

hipError_t mdlstm_forward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths, float* y,
                          unsigned long long* halo, unsigned* err, const float* x1, const float* const* W1,
                          const float* const* b1) {
  if (!mdlstm_supported(s)) return hipErrorInvalidValue;
  MdParams p = md_params(s, dirs, widths);
  p.y = y; p.halo = halo; p.err = err;
  const bool xin = x1 != nullptr;
  if (xin) {
    p.x = x1;
    for (int d = 0; d < 4; ++d) { p.W[d] = W1[d]; p.bias[d] = b1[d]; }
  }
  hipError_t e = md_clear(stream, s, halo, err, 64);
  if (e != hipSuccess) return e;
  const bool vec = md_vec(s, dirs, y);
  const int grid = 4 * s.B * p.NB;
  const bool xstage = xin && md_lds_fwd(2) + md_lds_xstage(s.Ww) <= (size_t)96 * 1024;
  const size_t xlds = xstage ? md_lds_xstage(s.Ww) : 0;
#define RLSTM_MD_FWD(HT_, VEC_, XIN_) \
  (!(XIN_) ? md_launch(mdlstm_fwd_kernel<HT_, VEC_, 0>, grid, 64 * (5 * HT_ + 2), md_lds_fwd(HT_), stream, p)                \
   : !xstage ? md_launch(mdlstm_fwd_kernel<HT_, VEC_, 1>, grid, 64 * (5 * HT_ + 2), md_lds_fwd(HT_), stream, p)              \
             : md_launch(mdlstm_fwd_kernel<HT_, VEC_, 2>, grid, 64 * (5 * HT_ + 2), md_lds_fwd(HT_) + xlds, stream, p))
  if (s.H <= 16) {
    if (xin) return vec ? RLSTM_MD_FWD(1, true, true) : RLSTM_MD_FWD(1, false, true);
    return vec ? RLSTM_MD_FWD(1, true, false) : RLSTM_MD_FWD(1, false, false);
  }
  if (xin) return vec ? RLSTM_MD_FWD(2, true, true) : RLSTM_MD_FWD(2, false, true);
  return vec ? RLSTM_MD_FWD(2, true, false) : RLSTM_MD_FWD(2, false, false);
#undef RLSTM_MD_FWD
}

size_t mdlstm_dbpart_floats(const MdShape& s) { return (size_t)4 * s.B * kMaxBands * 5 * s.H; }

hipError_t mdlstm_copy_x(hipStream_t stream, const MdShape& s, const MdDir* dirs, const float* x, int D) {
  MdXCopyParams q{};
  for (int d = 0; d < 4; ++d) q.hc[d] = dirs[d].hc;
  q.x = x; q.P = (size_t)s.Hh * s.Ww * s.B; q.D = D; q.H = s.H; q.S = s.S;
  const size_t total = q.P * D;
  hipLaunchKernelGGL(mdlstm_xcopy_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, q);
  return hipGetLastError();
}

hipError_t mdlstm_scatter_grads(hipStream_t stream, int D, int H, const float* const* stacked, float* const* dRu,
                                float* const* dRv, float* const* dW) {
  MdScatterParams q{};
  for (int d = 0; d < 4; ++d) { q.stacked[d] = stacked[d]; q.dRu[d] = dRu[d]; q.dRv[d] = dRv[d]; q.dW[d] = dW[d]; }
  q.D = D; q.H = H;
  const int total = (2 * H + D) * 5 * H;
  hipLaunchKernelGGL(mdlstm_scatter_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, q);
  return hipGetLastError();
}

hipError_t mdlstm_backward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths, const float* dy,
                           float* dbpart, float* const* db, unsigned long long* halo, unsigned* err) {
  if (!mdlstm_supported(s)) return hipErrorInvalidValue;
  MdParams p = md_params(s, dirs, widths);
  p.dy = dy; p.dbpart = dbpart; p.halo = halo; p.err = err;
  hipError_t e = md_clear(stream, s, halo, nullptr, 192);
  if (e != hipSuccess) return e;
  const bool vec = md_vec(s, dirs, dy);
  // the scan's workgroups, then as many again (at most 128) that clear the padding
  const int nscan = 4 * s.B * p.NB;
  const int grid = nscan + std::min(128, std::max(1, s.Hh * s.B));
  if (s.H <= 16) e = vec ? md_launch(mdlstm_bwd_kernel<1, true>, grid, 64 * 8, md_lds_bwd(1), stream, p)
                         : md_launch(mdlstm_bwd_kernel<1, false>, grid, 64 * 8, md_lds_bwd(1), stream, p);
  else e = vec ? md_launch(mdlstm_bwd_kernel<2, true>, grid, 64 * 13, md_lds_bwd(2), stream, p)
               : md_launch(mdlstm_bwd_kernel<2, false>, grid, 64 * 13, md_lds_bwd(2), stream, p);
  if (e != hipSuccess) return e;
  MdDbParams q{};
  for (int d = 0; d < 4; ++d) q.db[d] = db[d];
  q.dbpart = dbpart; q.B = s.B; q.NB = p.NB; q.n = 5 * s.H;
  hipLaunchKernelGGL(mdlstm_db_sum_kernel, dim3((unsigned)((q.n + 63) / 64), 4), dim3(64), 0, stream, q);
  return hipGetLastError();
}

}  // namespace rlstm
