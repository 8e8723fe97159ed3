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
// [R_u ; R_v]^T, K = 10H, same row / lane assignment; the gate derivatives follow in registers.
// d a overwrites the gates in place; [h_up | h_left] of every pixel is kept from the forward pass
// so that d R_u and d R_v are one whole-image product each afterwards.
#include "rlstm_internal.h"

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
__device__ __forceinline__ bool md_wait_word(const unsigned long long* q, unsigned long long& w, int diag, unsigned* err) {
  unsigned n = 0;
  unsigned long long t0 = 0;
  while ((unsigned)(w >> 32) != (unsigned)(diag + 1)) {
    w = md_ld_word(q);
    if ((++n & 255u) == 0) {
      const unsigned long long now = wall_clock64();
      if (t0 == 0) t0 = now;
      else if (now - t0 > kMdWaitTicks) return false;
      if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) return false;
    }
  }
  return true;
}

// VEC: H is a multiple of 4, so every group of four units starts 16-byte aligned in all tensors.
// Workgroup = (band, direction, image); 2 row tiles x HT unit halves, one wavefront each.
// Forward scan.  One wavefront per (gate, 16 units): 5 * HT wavefronts.  A step's product
// a^T = [R_u ; R_v]^T [h_up | h_left]^T is then 16 MFMAs per wavefront instead of 80, and a lane applies one
// nonlinearity to its four units instead of five; the wavefronts of the output gate pick up the other four
// activated gates from LDS (same lane, one 16-byte read each) and do the cell update.  The lane's 16 matrix
// operands (its column of [R_u ; R_v] for its gate and unit) never change and stay in registers.
// XIN: the input has one value per pixel (grayscale images): the input part b + x W of the pre-activation is formed
// here from x and this lane's weights and biases instead of being read from zg, and x is written next to
// [h_up | h_left] for the weight-gradient product.
template <int HT, bool VEC, int XM>
__global__ __launch_bounds__(64 * (5 * HT + 1)) void mdlstm_fwd_kernel(MdParams p) {
  constexpr bool XIN = XM != 0;        // XM: 0 input part read from zg, 1 x read from HBM, 2 the band's x staged in LDS
  static_assert(kTiles == 1, "one 16-row tile per band");
  constexpr int NTH = 64 * (5 * HT + 1);   // one more wavefront takes the rows handed from the band above
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
  const bool is_halo = wave == 5 * HT;
  const int g = is_halo ? 5 : wave / HT, ht = wave % HT;     // gate (i, f_u, f_v, o, g) and group of 16 units of this wavefront
  const int lr = l16;                          // row inside the band
  const int r = kBand * band + lr;             // row of this lane
  const int jm = 16 * ht + l16;                // unit whose column this lane feeds to the MFMA (A operand row)
  const int j0 = 16 * ht + 4 * lq;             // first of the four units this lane holds (accumulator rows)
  const int nv = is_halo ? 0 : min(max(H - j0, 0), 4);       // how many of them exist
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
    ra[ks] = (!is_halo && kk < H && jm < H) ? R[(size_t)kk * 5 * H + g * H + jm] : 0.f;
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
  const bool takes = band > 0, gives = band < p.NB - 1;
  const unsigned long long* halo_in = takes ? p.halo + ((size_t)dn * (p.NB - 1) + (band - 1)) * ndiag * 64 : p.halo;
  unsigned long long* halo_out = gives ? p.halo + ((size_t)dn * (p.NB - 1) + band) * ndiag * 64 : p.halo;
  const bool hands = is_halo && lane < HW;     // the lanes that move the handed row in
  const bool sends = wave == 1 && lane < HW;   // the lanes that hand this band's last row on (a wavefront that never loads)

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
      good = md_wait_word(halo_in + (size_t)sd * 64 + lane, hw, sd, p.err);
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
    if (gives && sends)                // last row of the band to the band below
      md_st_word(halo_out + (size_t)s * 64 + lane, lane < HP ? hcur[kBand * LDH + lane] : ccur[kBand * LDH + lane - HP], s);
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


template <int HT, bool VEC>
__global__ __launch_bounds__(64 * kTiles * HT) void mdlstm_bwd_kernel(MdParams p) {
  constexpr int NTH = 64 * kTiles * HT;
  constexpr int HP = 16 * HT;
  constexpr int NG = 5 * HP;
  constexpr int KS = 2 * NG / 4;
  constexpr int LDT = HP + 8;          // LDS row stride of [R_u ; R_v]^T
  constexpr int LDZ = NG + 4;          // LDS row stride of the d a rows
  constexpr int LDH = HP + 1;
  constexpr int HW = NG + HP;          // words of a handed row: d a | f_u * d c~
  extern __shared__ __align__(16) float lds[];
  float* RT = lds;                                   // [2NG][LDT]: row k < NG: R_u[.][k]; else R_v[.][k - NG]
  float* dzb = RT + 2 * NG * LDT;                    // [kBand + 1][LDZ]: d a of the diagonal done last; entry kBand is the row below the band
  float* dcu = dzb + (kBand + 1) * LDZ;              // [2][kBand + 1][LDH]: f_u * d c~ of a diagonal's pixels; entry kBand: row below
  float* dcv = dcu + 2 * (kBand + 1) * LDH;          // same with f_v

  // bands below come first in the grid
  const int dn = blockIdx.x % (4 * p.B), band = p.NB - 1 - blockIdx.x / (4 * p.B);
  const int d = dn & 3, n = dn >> 2;
  const int du = (d & 2) ? -1 : 1, dv = (d & 1) ? -1 : 1;
  const int H = p.H, Hh = p.Hh;
  const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
  const int lr = 16 * ((tid >> 6) % kTiles) + l16;  // row inside the band
  const int r = kBand * band + lr;             // row of this lane
  const int jm = 16 * (tid / (64 * kTiles)) + l16;        // unit whose row of [R_u ; R_v]^T this lane feeds to the MFMA
  const int j0 = 16 * (tid / (64 * kTiles)) + 4 * lq;     // first of the four units this lane handles
  const int nv = min(max(H - j0, 0), 4);
  const int wn = min(max(p.widths[n], 0), p.Ww);
  const int rows_here = min(Hh - kBand * band, kBand);

  for (int idx = tid; idx < 2 * NG * HP; idx += NTH) {
    const int k = idx / HP, jo = idx % HP;
    const int kk = k % NG, g = kk / HP, jj = kk % HP;
    float v = 0.f;
    if (jj < H && jo < H) v = (k < NG ? p.Ru[d] : p.Rv[d])[(size_t)jo * 5 * H + g * H + jj];
    RT[k * LDT + jo] = v;
  }
  for (int idx = tid; idx < (kBand + 1) * LDZ; idx += NTH) dzb[idx] = 0.f;
  for (int idx = tid; idx < 2 * (kBand + 1) * LDH; idx += NTH) { dcu[idx] = 0.f; dcv[idx] = 0.f; }
  __syncthreads();

  float* zgd = p.zg[d];
  const float* cd = p.c[d];
  const int s_lo = kBand * band, s_hi = wn > 0 ? kBand * band + rows_here - 1 + wn - 1 : s_lo - 1;
  const int ndiag = Hh + p.Ww;
  // the row below the band (first row of the band below) has pixels on diagonals b_lo .. b_lo + wn - 1
  const int b_lo = kBand * (band + 1);
  const bool takes = band < p.NB - 1, gives = band > 0;
  const unsigned long long* halo_in = takes ? p.halo + ((size_t)dn * (p.NB - 1) + band) * ndiag * 192 : p.halo;
  unsigned long long* halo_out = gives ? p.halo + ((size_t)dn * (p.NB - 1) + (band - 1)) * ndiag * 192 : p.halo;

  // d a and f_u * d c~ of the row below on diagonal sd -> entry kBand of dzb / the given dcu buffer (wavefront 0)
  unsigned long long hw[3] = {0, 0, 0};
  auto halo_issue = [&](int sd) {
    if (tid < 64 && takes && sd >= b_lo && sd <= b_lo + wn - 1)
#pragma unroll
      for (int k = 0; k < 3; ++k)
        if (tid + 64 * k < HW) hw[k] = md_ld_word(halo_in + (size_t)sd * 192 + tid + 64 * k);
  };
  auto halo_take = [&](int sd, float* dcu_dst) -> bool {
    if (tid >= 64) return true;
    bool good = true;
    const bool have = takes && sd >= b_lo && sd <= b_lo + wn - 1;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int w = tid + 64 * k;
      if (w >= HW) continue;
      float v = 0.f;
      if (have) {
        good = md_wait_word(halo_in + (size_t)sd * 192 + w, hw[k], sd, p.err) && good;
        v = __uint_as_float((unsigned)hw[k]);
      }
      if (w < NG) dzb[kBand * LDZ + w] = v; else dcu_dst[kBand * LDH + w - NG] = v;
    }
    return good;
  };

  // bias gradient of the lane's four units, summed over all diagonals
  floatx4 dbacc[5];
#pragma unroll
  for (int g = 0; g < 5; ++g) dbacc[g] = floatx4{0.f, 0.f, 0.f, 0.f};

  // gates, c, c of the two predecessors and dy of the lane's row and four units on diagonal s
  floatx4 in[9];
  auto prefetch = [&](int s) {
    const int q = s - r;
    const bool ok = s >= s_lo && lr < rows_here && q >= 0 && q < wn && nv > 0;
    const floatx4 zero = floatx4{0.f, 0.f, 0.f, 0.f};
    const size_t pix = ok ? md_pixel(p, du, dv, wn, n, r, q) : 0;
#pragma unroll
    for (int g = 0; g < 5; ++g) in[g] = ok ? ld4<VEC>(zgd + pix * 5 * H + g * H + j0, nv) : zero;
    in[5] = ok ? ld4<VEC>(cd + pix * H + j0, nv) : zero;
    in[6] = (ok && r >= 1) ? ld4<VEC>(cd + md_pixel(p, du, dv, wn, n, r - 1, q) * H + j0, nv) : zero;
    in[7] = (ok && q >= 1) ? ld4<VEC>(cd + md_pixel(p, du, dv, wn, n, r, q - 1) * H + j0, nv) : zero;
    in[8] = ok ? ld4<VEC>(p.dy + pix * 4 * H + d * H + j0, nv) : zero;
  };
  prefetch(s_hi);
  int fail = 0;
  {
    // the row below on the diagonal after the last one
    halo_issue(s_hi + 1);
    if (!halo_take(s_hi + 1, dcu + ((s_hi + 1) & 1) * (kBand + 1) * LDH)) fail = 1;
  }
  if (__syncthreads_or(fail)) {
    if (tid == 0) __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return;
  }

  // this lane's A operands of every MFMA of a step: they do not change from diagonal to diagonal
  float rt[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) rt[ks] = RT[(4 * ks + lq) * LDT + jm];

  for (int s = s_hi; s >= s_lo; --s) {
    const float* dcu_prev = dcu + ((s + 1) & 1) * (kBand + 1) * LDH;
    const float* dcv_prev = dcv + ((s + 1) & 1) * (kBand + 1) * LDH;
    float* dcu_cur = dcu + (s & 1) * (kBand + 1) * LDH;
    float* dcv_cur = dcv + (s & 1) * (kBand + 1) * LDH;
    if (s > s_lo) halo_issue(s);       // arrives while the MFMAs run

    // d h^T of diagonal s = [R_u ; R_v] [d a(row + 1) | d a(row)]^T of diagonal s+1 (the successor below sits in
    // row r+1, the one to the right in row r); two accumulators so that consecutive MFMAs do not wait for each other
    floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = floatx4{0.f, 0.f, 0.f, 0.f};
    const float* brow = dzb + lr * LDZ;
#pragma unroll
    for (int ks = 0; ks < KS; ks += 2) {
      const int k0 = 4 * ks + lq, k1 = k0 + 4;
      const float b0 = k0 < NG ? brow[LDZ + k0] : brow[k0 - NG];
      const float b1 = k1 < NG ? brow[LDZ + k1] : brow[k1 - NG];
      acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(rt[ks], b0, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(rt[ks + 1], b1, acc1, 0, 0, 0);
    }
    const floatx4 acc = acc0 + acc1;
    __syncthreads();     // every wavefront has read the d a rows of diagonal s+1

    const int q = s - r;
    const bool ok = lr < rows_here && q >= 0 && q < wn && nv > 0;
    const size_t pix = ok ? md_pixel(p, du, dv, wn, n, r, q) : 0;
    floatx4 dz[5];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = j0 + i;
      const bool oki = ok && i < nv;
      const float gi = in[0][i], gfu = in[1][i], gfv = in[2][i], go = in[3][i], gg = in[4][i];
      const float tc = md_tanh(in[5][i]);
      const float dh = in[8][i] + acc[i];
      const float d_o = dh * tc;
      const float dct = dcu_prev[(lr + 1) * LDH + j] + dcv_prev[lr * LDH + j] + dh * go * (1.0f - tc * tc);
      dz[0][i] = oki ? dct * gg * gi * (1.0f - gi) : 0.f;
      dz[1][i] = oki ? dct * in[6][i] * gfu * (1.0f - gfu) : 0.f;
      dz[2][i] = oki ? dct * in[7][i] * gfv * (1.0f - gfv) : 0.f;
      dz[3][i] = oki ? d_o * go * (1.0f - go) : 0.f;
      dz[4][i] = oki ? dct * gi * (1.0f - gg * gg) : 0.f;
      dcu_cur[lr * LDH + j] = oki ? dct * gfu : 0.f;
      dcv_cur[lr * LDH + j] = oki ? dct * gfv : 0.f;
#pragma unroll
      for (int g = 0; g < 5; ++g) dzb[lr * LDZ + g * HP + j] = dz[g][i];
    }
#pragma unroll
    for (int g = 0; g < 5; ++g) dbacc[g] += dz[g];
    // the row below on this diagonal, for the next step
    fail = (s > s_lo ? halo_take(s, dcu_cur) : true) ? 0 : 1;
    // the LDS rows of diagonal s are complete; HBM traffic follows the barrier
    if (__syncthreads_or(fail)) {
      if (tid == 0) __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return;
    }
    if (gives && tid < 64) {           // first row of the band to the band above
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const int w = tid + 64 * k;
        if (w < HW) md_st_word(halo_out + (size_t)s * 192 + w, w < NG ? dzb[w] : dcu_cur[w - NG], s);
      }
    }
    if (ok) {
      float* zrow = zgd + pix * 5 * H + j0;
#pragma unroll
      for (int g = 0; g < 5; ++g) st4<VEC>(zrow + g * H, dz[g], nv);
    }
    prefetch(s - 1);
  }
  __syncthreads();

  // bias gradient of this (direction, image, band): the threads that share a unit are added in thread order
  float* stage = dzb;                                // [threads][5][4]
#pragma unroll
  for (int g = 0; g < 5; ++g)
#pragma unroll
    for (int i = 0; i < 4; ++i) stage[(tid * 5 + g) * 4 + i] = dbacc[g][i];
  __syncthreads();
  for (int idx = tid; idx < 5 * HP; idx += NTH) {
    const int g = idx / HP, jo = idx % HP;
    if (jo < H) {
      // threads that handle unit jo: unit half jo / 16, quad (jo % 16) / 4, every row tile and row lane
      float sum = 0.f;
      for (int w = 0; w < kTiles; ++w)
        for (int l = 0; l < 16; ++l)
          sum += stage[((64 * kTiles * (jo >> 4) + 64 * w + 16 * ((jo & 15) >> 2) + l) * 5 + g) * 4 + (jo & 3)];
      p.dbpart[((size_t)dn * p.NB + band) * 5 * H + g * H + jo] = sum;
    }
  }

  // d a = 0 beyond the image's width
  const int npad = (p.Ww - wn) * rows_here;
  for (int idx = tid; idx < npad * 5 * H; idx += NTH) {
    const int col = idx % (5 * H), cell = idx / (5 * H);
    const int rr = kBand * band + cell / (p.Ww - wn), v = wn + cell % (p.Ww - wn);
    const int u = du > 0 ? rr : Hh - 1 - rr;
    const size_t pix = ((size_t)u * p.Ww + v) * p.B + n;
    zgd[pix * 5 * H + col] = 0.f;
  }
}

// db[d][col] = sum over the images and their bands, in that order
struct MdDbParams { float* db[4]; const float* dbpart; int B, NB, n; };
__global__ __launch_bounds__(256) void mdlstm_db_sum_kernel(MdDbParams p) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= p.n) return;
  for (int d = 0; d < 4; ++d) {
    float sum = 0.f;
    for (int b = 0; b < p.B; ++b)
      for (int k = 0; k < p.NB; ++k) sum += p.dbpart[((size_t)(b * 4 + d) * p.NB + k) * p.n + i];
    p.db[d][i] = sum;
  }
}

// clears the handed-row words and the timeout flag before a pass
__global__ __launch_bounds__(256) void mdlstm_clear_kernel(unsigned long long* words, size_t n, unsigned* err) {
  const size_t gsz = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += gsz) words[i] = 0ull;
  if (blockIdx.x == 0 && threadIdx.x == 0) *err = 0u;
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
  return ((size_t)2 * NG * (HP + 8) + (size_t)(kBand + 1) * (NG + 4) + (size_t)4 * (kBand + 1) * (HP + 1)) * sizeof(float);
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

MdParams md_params(const MdShape& s, const MdDir* dirs, const int32_t* widths) {
  MdParams p{};
  for (int d = 0; d < 4; ++d) {
    p.zg[d] = dirs[d].zg; p.c[d] = dirs[d].c; p.hc[d] = dirs[d].hc; p.Ru[d] = dirs[d].Ru; p.Rv[d] = dirs[d].Rv;
  }
  p.widths = widths; p.Hh = s.Hh; p.Ww = s.Ww; p.B = s.B; p.H = s.H; p.S = s.S;
  p.NB = (s.Hh + kBand - 1) / kBand;
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
  (!(XIN_) ? md_launch(mdlstm_fwd_kernel<HT_, VEC_, 0>, grid, 64 * (5 * HT_ + 1), md_lds_fwd(HT_), stream, p)                \
   : !xstage ? md_launch(mdlstm_fwd_kernel<HT_, VEC_, 1>, grid, 64 * (5 * HT_ + 1), md_lds_fwd(HT_), stream, p)              \
             : md_launch(mdlstm_fwd_kernel<HT_, VEC_, 2>, grid, 64 * (5 * HT_ + 1), md_lds_fwd(HT_) + xlds, stream, p))
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
  hipError_t e = md_clear(stream, s, halo, err, 192);
  if (e != hipSuccess) return e;
  const bool vec = md_vec(s, dirs, dy);
  const int grid = 4 * s.B * p.NB;
  if (s.H <= 16) e = vec ? md_launch(mdlstm_bwd_kernel<1, true>, grid, 64 * kTiles, md_lds_bwd(1), stream, p)
                         : md_launch(mdlstm_bwd_kernel<1, false>, grid, 64 * kTiles, md_lds_bwd(1), stream, p);
  else e = vec ? md_launch(mdlstm_bwd_kernel<2, true>, grid, 128 * kTiles, md_lds_bwd(2), stream, p)
               : md_launch(mdlstm_bwd_kernel<2, false>, grid, 128 * kTiles, md_lds_bwd(2), stream, p);
  if (e != hipSuccess) return e;
  MdDbParams q{};
  for (int d = 0; d < 4; ++d) q.db[d] = db[d];
  q.dbpart = dbpart; q.B = s.B; q.NB = p.NB; q.n = 5 * s.H;
  hipLaunchKernelGGL(mdlstm_db_sum_kernel, dim3((unsigned)((q.n + 255) / 256)), dim3(256), 0, stream, q);
  return hipGetLastError();
}

}  // namespace rlstm
