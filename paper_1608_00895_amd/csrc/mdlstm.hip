// Two-dimensional LSTM layer (Sec. 4.2 of the RETURNN paper): the hidden state of pixel (u, v)
// needs the states of (u-1, v) and (u, v-1) in scan order, so all pixels of one anti-diagonal can
// be computed together; four scan directions and several images run at once.
//
// One workgroup (4 wavefronts per 16 units) per (scan direction, image); it walks the anti-diagonals of its
// image from the first pixel of the scan to the last, at the image's own width, so images of a
// batch never wait for each other and nothing is exchanged between workgroups.  In scan
// coordinates (row r = 0 .. Hh-1, column q = 0 .. width-1) diagonal s holds the pixels r + q = s;
// the pixel of row r on diagonal s has its vertical predecessor in row r-1 and its horizontal
// predecessor in row r, both on diagonal s-1.  The workgroup keeps h and c of the previous
// diagonal in LDS, indexed by row (rows without a pixel hold zeros, which is also what a
// predecessor outside the image contributes), and the recurrent matrices [R_u ; R_v] in LDS for
// the whole scan.
//
// Forward step: [64 rows x 2H] * [2H x 5H] on the matrix cores (v_mfma_f32_16x16x4_f32; a wavefront
// owns rows 16w .. 16w+15 and the five gate columns of 16 units, so the five gate pre-activations of
// a (row, unit) pair end up in one lane and the gating needs no exchange; with 32 units two
// wavefronts share a SIMD and one's gating overlaps the other's MFMAs), plus the input part
// X W + b that a whole-image product wrote beforehand, prefetched one diagonal ahead.
// Backward step (diagonals in reverse): d h = [d a(r+1) | d a(r)] of diagonal s+1 times
// [R_u ; R_v]^T, K = 10H, same row / lane assignment; the gate derivatives follow in registers.
// d a overwrites the gates in place; [h_up | h_left] of every pixel is kept from the forward pass
// so that d R_u and d R_v are one whole-image product each afterwards.
#include "rlstm_internal.h"

namespace rlstm {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kRows = 64;      // image rows a workgroup holds (4 wavefronts x one 16-row MFMA tile)

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
  float* dbpart;           // backward: [4][B][5H] bias gradient of every (direction, image)
  const int32_t* widths;   // [B]
  int Hh, Ww, B, H, S;
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

// VEC: H is a multiple of 4, so every group of four units starts 16-byte aligned in all tensors
template <int HT, bool VEC>
__global__ __launch_bounds__(256 * HT) void mdlstm_fwd_kernel(MdParams p) {
  constexpr int NTH = 256 * HT;        // threads: 4 row tiles x HT unit halves, one wavefront each
  constexpr int HP = 16 * HT;          // padded units
  constexpr int NG = 5 * HP;           // padded pre-activation width
  constexpr int KS = 2 * HP / 4;       // MFMA k-steps
  constexpr int LDR = NG + 8;          // LDS row stride of [R_u ; R_v] (rows 4 apart fall into different banks)
  constexpr int LDH = HP + 1;
  extern __shared__ __align__(16) float lds[];
  float* Rs = lds;                                   // [2HP][LDR]
  float* hb = Rs + 2 * HP * LDR;                     // [2][kRows + 1][LDH]; entry 0 is row -1 and stays zero
  float* cb = hb + 2 * (kRows + 1) * LDH;            // same for c

  const int d = blockIdx.x & 3, n = blockIdx.x >> 2;
  const int du = (d & 2) ? -1 : 1, dv = (d & 1) ? -1 : 1;
  const int H = p.H, Hh = p.Hh;
  const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
  const int wave = (tid >> 6) & 3;     // row tile
  const int r = 16 * wave + l16;       // row of this lane
  const int jm = 16 * (tid >> 8) + l16;        // unit whose columns this lane feeds to the MFMA (A operand row)
  const int j0 = 16 * (tid >> 8) + 4 * lq;     // first of the four units this lane gates (accumulator rows)
  const int nv = min(max(H - j0, 0), 4);       // how many of them exist
  const int wn = min(max(p.widths[n], 0), p.Ww);

  for (int idx = tid; idx < 2 * HP * NG; idx += NTH) {
    const int k = idx / NG, col = idx % NG;
    const int g = col / HP, jj = col % HP, kk = k % HP;
    float v = 0.f;
    if (kk < H && jj < H) v = (k < HP ? p.Ru[d] : p.Rv[d])[(size_t)kk * 5 * H + g * H + jj];
    Rs[k * LDR + col] = v;
  }
  for (int idx = tid; idx < 2 * (kRows + 1) * LDH; idx += NTH) { hb[idx] = 0.f; cb[idx] = 0.f; }
  __syncthreads();

  float* zgd = p.zg[d];
  float* cd = p.c[d];
  float* hcd = p.hc[d];
  const int nsteps = wn > 0 ? Hh + wn - 1 : 0;

  // input part of the lane's row and four units on diagonal s
  floatx4 zr[5];
  auto prefetch = [&](int s) {
    const int q = s - r;
    const bool ok = r < Hh && q >= 0 && q < wn && s < nsteps && nv > 0;
    const size_t pix = ok ? md_pixel(p, du, dv, wn, n, r, q) : 0;
#pragma unroll
    for (int g = 0; g < 5; ++g)
      zr[g] = ok ? ld4<VEC>(zgd + pix * 5 * H + g * H + j0, nv) : floatx4{0.f, 0.f, 0.f, 0.f};
  };
  prefetch(0);

  for (int s = 0; s < nsteps; ++s) {
    const float* hprev = hb + ((s + 1) & 1) * (kRows + 1) * LDH;
    const float* cprev = cb + ((s + 1) & 1) * (kRows + 1) * LDH;
    float* hcur = hb + (s & 1) * (kRows + 1) * LDH;
    float* ccur = cb + (s & 1) * (kRows + 1) * LDH;

    // a^T = [R_u ; R_v]^T [h_up | h_left]^T: accumulator g holds gate g of units j0 .. j0+3 (its 4 rows) for the
    // image row of this lane (its column).  A[m][k] = R[k][gate column of unit jm]; B[k][n]: k < HP: h of the
    // row above (entry index = row), else h of the same row (entry index row + 1)
    floatx4 acc[5];
#pragma unroll
    for (int g = 0; g < 5; ++g) acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
    const float* brow = hprev + r * LDH;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k = 4 * ks + lq;
      const float hv = k < HP ? brow[k] : brow[LDH + k - HP];
#pragma unroll
      for (int g = 0; g < 5; ++g)
        acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(Rs[k * LDR + g * HP + jm], hv, acc[g], 0, 0, 0);
    }

    const int q = s - r;
    const bool ok = r < Hh && q >= 0 && q < wn && nv > 0;
    const size_t pix = ok ? md_pixel(p, du, dv, wn, n, r, q) : 0;
    floatx4 gi, gfu, gfv, go, gg, ct, ht, h_up, h_left;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = j0 + i;
      gi[i] = md_sigmoid(acc[0][i] + zr[0][i]);
      gfu[i] = md_sigmoid(acc[1][i] + zr[1][i]);
      gfv[i] = md_sigmoid(acc[2][i] + zr[2][i]);
      go[i] = md_sigmoid(acc[3][i] + zr[3][i]);
      gg[i] = md_tanh(acc[4][i] + zr[4][i]);
      h_up[i] = hprev[r * LDH + j]; h_left[i] = hprev[(r + 1) * LDH + j];
      const float c_up = cprev[r * LDH + j], c_left = cprev[(r + 1) * LDH + j];
      ct[i] = gfu[i] * c_up + gfv[i] * c_left + gi[i] * gg[i];
      ht[i] = go[i] * md_tanh(ct[i]);
      const bool oki = ok && i < nv;
      hcur[(r + 1) * LDH + j] = oki ? ht[i] : 0.f;
      ccur[(r + 1) * LDH + j] = oki ? ct[i] : 0.f;
    }
    // the next diagonal only needs the LDS rows: the stores to HBM and the next prefetch follow the barrier, so
    // that one wavefront's memory instructions overlap the MFMAs of the wavefront it shares the SIMD with
    __syncthreads();
    if (ok) {
      float* zrow = zgd + pix * 5 * H + j0;
      st4<VEC>(zrow, gi, nv); st4<VEC>(zrow + H, gfu, nv); st4<VEC>(zrow + 2 * H, gfv, nv);
      st4<VEC>(zrow + 3 * H, go, nv); st4<VEC>(zrow + 4 * H, gg, nv);
      st4<VEC>(cd + pix * H + j0, ct, nv);
      st4<VEC>(p.y + pix * 4 * H + d * H + j0, ht, nv);
      st4<VEC>(hcd + pix * p.S + j0, h_up, nv);
      st4<VEC>(hcd + pix * p.S + H + j0, h_left, nv);
    }
    prefetch(s + 1);
  }

  // pixels beyond the image's width: y = 0, and zeros where the products after the backward pass read
  const int npad = (p.Ww - wn) * Hh;
  for (int idx = tid; idx < npad * H; idx += NTH) {
    const int jj = idx % H, cell = idx / H;
    const int u = cell / (p.Ww - wn), v = wn + cell % (p.Ww - wn);
    const size_t pix = ((size_t)u * p.Ww + v) * p.B + n;
    p.y[pix * 4 * H + d * H + jj] = 0.f;
    cd[pix * H + jj] = 0.f;
    hcd[pix * p.S + jj] = 0.f;
    hcd[pix * p.S + H + jj] = 0.f;
  }
}

template <int HT, bool VEC>
__global__ __launch_bounds__(256 * HT) void mdlstm_bwd_kernel(MdParams p) {
  constexpr int NTH = 256 * HT;
  constexpr int HP = 16 * HT;
  constexpr int NG = 5 * HP;
  constexpr int KS = 2 * NG / 4;
  constexpr int LDT = HP + 8;          // LDS row stride of [R_u ; R_v]^T
  constexpr int LDZ = NG + 4;          // LDS row stride of the d a rows
  constexpr int LDH = HP + 1;
  extern __shared__ __align__(16) float lds[];
  float* RT = lds;                                   // [2NG][LDT]: row k < NG: R_u[.][k]; else R_v[.][k - NG]
  float* dzb = RT + 2 * NG * LDT;                    // [kRows + 1][LDZ]: d a of the diagonal done last; entry kRows stays zero
  float* dcu = dzb + (kRows + 1) * LDZ;              // [2][kRows + 1][LDH]: f_u * d c~ of a diagonal's pixels
  float* dcv = dcu + 2 * (kRows + 1) * LDH;          // same with f_v

  const int d = blockIdx.x & 3, n = blockIdx.x >> 2;
  const int du = (d & 2) ? -1 : 1, dv = (d & 1) ? -1 : 1;
  const int H = p.H, Hh = p.Hh;
  const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
  const int wave = (tid >> 6) & 3;     // row tile
  const int r = 16 * wave + l16;       // row of this lane
  const int jm = 16 * (tid >> 8) + l16;        // unit whose row of [R_u ; R_v]^T this lane feeds to the MFMA
  const int j0 = 16 * (tid >> 8) + 4 * lq;     // first of the four units this lane handles
  const int nv = min(max(H - j0, 0), 4);
  const int wn = min(max(p.widths[n], 0), p.Ww);

  for (int idx = tid; idx < 2 * NG * HP; idx += NTH) {
    const int k = idx / HP, jo = idx % HP;
    const int kk = k % NG, g = kk / HP, jj = kk % HP;
    float v = 0.f;
    if (jj < H && jo < H) v = (k < NG ? p.Ru[d] : p.Rv[d])[(size_t)jo * 5 * H + g * H + jj];
    RT[k * LDT + jo] = v;
  }
  for (int idx = tid; idx < (kRows + 1) * LDZ; idx += NTH) dzb[idx] = 0.f;
  for (int idx = tid; idx < 2 * (kRows + 1) * LDH; idx += NTH) { dcu[idx] = 0.f; dcv[idx] = 0.f; }
  __syncthreads();

  float* zgd = p.zg[d];
  const float* cd = p.c[d];
  const int nsteps = wn > 0 ? Hh + wn - 1 : 0;

  // bias gradient of the lane's four units, summed over all diagonals
  floatx4 dbacc[5];
#pragma unroll
  for (int g = 0; g < 5; ++g) dbacc[g] = floatx4{0.f, 0.f, 0.f, 0.f};

  // gates, c, c of the two predecessors and dy of the lane's row and four units on diagonal s
  floatx4 in[9];
  auto prefetch = [&](int s) {
    const int q = s - r;
    const bool ok = s >= 0 && r < Hh && q >= 0 && q < wn && nv > 0;
    const floatx4 zero = floatx4{0.f, 0.f, 0.f, 0.f};
    const size_t pix = ok ? md_pixel(p, du, dv, wn, n, r, q) : 0;
#pragma unroll
    for (int g = 0; g < 5; ++g) in[g] = ok ? ld4<VEC>(zgd + pix * 5 * H + g * H + j0, nv) : zero;
    in[5] = ok ? ld4<VEC>(cd + pix * H + j0, nv) : zero;
    in[6] = (ok && r >= 1) ? ld4<VEC>(cd + md_pixel(p, du, dv, wn, n, r - 1, q) * H + j0, nv) : zero;
    in[7] = (ok && q >= 1) ? ld4<VEC>(cd + md_pixel(p, du, dv, wn, n, r, q - 1) * H + j0, nv) : zero;
    in[8] = ok ? ld4<VEC>(p.dy + pix * 4 * H + d * H + j0, nv) : zero;
  };
  prefetch(nsteps - 1);

  for (int s = nsteps - 1; s >= 0; --s) {
    const float* dcu_prev = dcu + ((s + 1) & 1) * (kRows + 1) * LDH;
    const float* dcv_prev = dcv + ((s + 1) & 1) * (kRows + 1) * LDH;
    float* dcu_cur = dcu + (s & 1) * (kRows + 1) * LDH;
    float* dcv_cur = dcv + (s & 1) * (kRows + 1) * LDH;

    // d h^T of diagonal s = [R_u ; R_v] [d a(row + 1) | d a(row)]^T of diagonal s+1 (the successor below sits in
    // row r+1, the one to the right in row r); two accumulators so that consecutive MFMAs do not wait for each other
    floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = floatx4{0.f, 0.f, 0.f, 0.f};
    const float* brow = dzb + r * LDZ;
#pragma unroll 8
    for (int ks = 0; ks < KS; ks += 2) {
      const int k0 = 4 * ks + lq, k1 = k0 + 4;
      const float b0 = k0 < NG ? brow[LDZ + k0] : brow[k0 - NG];
      const float b1 = k1 < NG ? brow[LDZ + k1] : brow[k1 - NG];
      acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(RT[k0 * LDT + jm], b0, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(RT[k1 * LDT + jm], b1, acc1, 0, 0, 0);
    }
    const floatx4 acc = acc0 + acc1;
    __syncthreads();     // every wavefront has read the d a rows of diagonal s+1

    const int q = s - r;
    const bool ok = r < Hh && q >= 0 && q < wn && nv > 0;
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
      const float dct = dcu_prev[(r + 1) * LDH + j] + dcv_prev[r * LDH + j] + dh * go * (1.0f - tc * tc);
      dz[0][i] = oki ? dct * gg * gi * (1.0f - gi) : 0.f;
      dz[1][i] = oki ? dct * in[6][i] * gfu * (1.0f - gfu) : 0.f;
      dz[2][i] = oki ? dct * in[7][i] * gfv * (1.0f - gfv) : 0.f;
      dz[3][i] = oki ? d_o * go * (1.0f - go) : 0.f;
      dz[4][i] = oki ? dct * gi * (1.0f - gg * gg) : 0.f;
      dcu_cur[r * LDH + j] = oki ? dct * gfu : 0.f;
      dcv_cur[r * LDH + j] = oki ? dct * gfv : 0.f;
#pragma unroll
      for (int g = 0; g < 5; ++g) dzb[r * LDZ + g * HP + j] = dz[g][i];
    }
#pragma unroll
    for (int g = 0; g < 5; ++g) dbacc[g] += dz[g];
    __syncthreads();     // the LDS rows of diagonal s are complete; HBM traffic follows the barrier
    if (ok) {
      float* zrow = zgd + pix * 5 * H + j0;
#pragma unroll
      for (int g = 0; g < 5; ++g) st4<VEC>(zrow + g * H, dz[g], nv);
    }
    prefetch(s - 1);
  }
  __syncthreads();

  // bias gradient of this (direction, image): the 16 threads that share a unit are added in thread order
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
      for (int w = 0; w < 4; ++w)
        for (int l = 0; l < 16; ++l)
          sum += stage[((256 * (jo >> 4) + 64 * w + 16 * ((jo & 15) >> 2) + l) * 5 + g) * 4 + (jo & 3)];
      p.dbpart[((size_t)d * p.B + n) * 5 * H + g * H + jo] = sum;
    }
  }

  // d a = 0 beyond the image's width
  const int npad = (p.Ww - wn) * Hh;
  for (int idx = tid; idx < npad * 5 * H; idx += NTH) {
    const int col = idx % (5 * H), cell = idx / (5 * H);
    const int u = cell / (p.Ww - wn), v = wn + cell % (p.Ww - wn);
    const size_t pix = ((size_t)u * p.Ww + v) * p.B + n;
    zgd[pix * 5 * H + col] = 0.f;
  }
}

// db[d][col] = sum over the images, in image order
struct MdDbParams { float* db[4]; const float* dbpart; int B, n; };
__global__ __launch_bounds__(256) void mdlstm_db_sum_kernel(MdDbParams p) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= p.n) return;
  for (int d = 0; d < 4; ++d) {
    float sum = 0.f;
    for (int b = 0; b < p.B; ++b) sum += p.dbpart[((size_t)d * p.B + b) * p.n + i];
    p.db[d][i] = sum;
  }
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
  const int HP = 16 * HT, NG = 5 * HP;
  return ((size_t)2 * HP * (NG + 8) + (size_t)4 * (kRows + 1) * (HP + 1)) * sizeof(float);
}
size_t md_lds_bwd(int HT) {
  const int HP = 16 * HT, NG = 5 * HP;
  return ((size_t)2 * NG * (HP + 8) + (size_t)(kRows + 1) * (NG + 4) + (size_t)4 * (kRows + 1) * (HP + 1)) * sizeof(float);
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

bool mdlstm_supported(const MdShape& s) { return s.Hh >= 1 && s.Hh <= kRows && s.H >= 1 && s.H <= 32; }

hipError_t mdlstm_forward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths, float* y) {
  if (!mdlstm_supported(s)) return hipErrorInvalidValue;
  MdParams p = md_params(s, dirs, widths);
  p.y = y;
  const bool vec = md_vec(s, dirs, y);
  if (s.H <= 16) return vec ? md_launch(mdlstm_fwd_kernel<1, true>, 4 * s.B, 256, md_lds_fwd(1), stream, p)
                            : md_launch(mdlstm_fwd_kernel<1, false>, 4 * s.B, 256, md_lds_fwd(1), stream, p);
  return vec ? md_launch(mdlstm_fwd_kernel<2, true>, 4 * s.B, 512, md_lds_fwd(2), stream, p)
             : md_launch(mdlstm_fwd_kernel<2, false>, 4 * s.B, 512, md_lds_fwd(2), stream, p);
}

size_t mdlstm_dbpart_floats(const MdShape& s) { return (size_t)4 * s.B * 5 * s.H; }

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
                           float* dbpart, float* const* db) {
  if (!mdlstm_supported(s)) return hipErrorInvalidValue;
  MdParams p = md_params(s, dirs, widths);
  p.dy = dy;
  p.dbpart = dbpart;
  const bool vec = md_vec(s, dirs, dy);
  hipError_t e;
  if (s.H <= 16) e = vec ? md_launch(mdlstm_bwd_kernel<1, true>, 4 * s.B, 256, md_lds_bwd(1), stream, p)
                         : md_launch(mdlstm_bwd_kernel<1, false>, 4 * s.B, 256, md_lds_bwd(1), stream, p);
  else e = vec ? md_launch(mdlstm_bwd_kernel<2, true>, 4 * s.B, 512, md_lds_bwd(2), stream, p)
               : md_launch(mdlstm_bwd_kernel<2, false>, 4 * s.B, 512, md_lds_bwd(2), stream, p);
  if (e != hipSuccess) return e;
  MdDbParams q{};
  for (int d = 0; d < 4; ++d) q.db[d] = db[d];
  q.dbpart = dbpart; q.B = s.B; q.n = 5 * s.H;
  hipLaunchKernelGGL(mdlstm_db_sum_kernel, dim3((unsigned)((q.n + 255) / 256)), dim3(256), 0, stream, q);
  return hipGetLastError();
}

}  // namespace rlstm
