// Two-dimensional LSTM layer (Sec. 4.2 of the RETURNN paper): the hidden state of pixel (u, v)
// needs the states of (u-1, v) and (u, v-1) in scan order, so all pixels of one anti-diagonal can
// be computed together; four scan directions and several images run at once.
//
// One workgroup (4 wavefronts) per (scan direction, image); it walks the anti-diagonals of its
// image from the first pixel of the scan to the last, at the image's own width, so images of a
// batch never wait for each other and nothing is exchanged between workgroups.  In scan
// coordinates (row r = 0 .. Hh-1, column q = 0 .. width-1) diagonal s holds the pixels r + q = s;
// the pixel of row r on diagonal s has its vertical predecessor in row r-1 and its horizontal
// predecessor in row r, both on diagonal s-1.  The workgroup keeps h and c of the previous
// diagonal in LDS, indexed by row (rows without a pixel hold zeros, which is also what a
// predecessor outside the image contributes), and the recurrent matrices [R_u ; R_v] in LDS for
// the whole scan.
//
// Forward step: [64 rows x 2H] * [2H x 5H] on the matrix cores (v_mfma_f32_16x16x4_f32; wavefront
// w owns rows 16w .. 16w+15 and all 5H columns, so the five gate pre-activations of a (row, unit)
// pair end up in one lane and the gating needs no exchange), plus the input part X W + b that a
// whole-image product wrote beforehand, prefetched one diagonal ahead.
// Backward step (diagonals in reverse): d h = [d a(r+1) | d a(r)] of diagonal s+1 times
// [R_u ; R_v]^T, K = 10H, same row / lane assignment; the gate derivatives follow in registers.
// d a overwrites the gates in place; [h_up | h_left] of every pixel is kept from the forward pass
// so that d R_u and d R_v are one whole-image product each afterwards.
#include "rlstm_internal.h"

namespace rlstm {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kRows = 64;      // image rows a workgroup holds (4 wavefronts x one 16-row MFMA tile)

__device__ __forceinline__ float md_sigmoid(float u) { return __builtin_amdgcn_rcpf(1.0f + expf(-u)); }
__device__ __forceinline__ float md_tanh(float u) { return 2.0f * __builtin_amdgcn_rcpf(1.0f + expf(-2.0f * u)) - 1.0f; }

struct MdParams {
  float* zg[4];            // [P, 5H]: X W + b -> gates i|f_u|f_v|o|g -> d a
  float* c[4];             // [P, H]
  float* hc[4];            // [P, 2H]: h_up | h_left of every pixel
  const float* Ru[4];      // [H, 5H]
  const float* Rv[4];
  float* y;                // forward: [P, 4H] output
  const float* dy;         // backward: [P, 4H]
  const int32_t* widths;   // [B]
  int Hh, Ww, B, H;
};

// scan coordinates (row r, column q) of image n, direction (du, dv), image width wn -> pixel index
__device__ __forceinline__ size_t md_pixel(const MdParams& p, int du, int dv, int wn, int n, int r, int q) {
  const int u = du > 0 ? r : p.Hh - 1 - r;
  const int v = dv > 0 ? q : wn - 1 - q;
  return ((size_t)u * p.Ww + v) * p.B + n;
}

template <int HT>
__global__ __launch_bounds__(256) void mdlstm_fwd_kernel(MdParams p) {
  constexpr int HP = 16 * HT;          // padded units
  constexpr int NG = 5 * HP;           // padded pre-activation width
  constexpr int NTL = 5 * HT;          // 16-column tiles
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
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
  const int wn = min(max(p.widths[n], 0), p.Ww);

  for (int idx = tid; idx < 2 * HP * NG; idx += 256) {
    const int k = idx / NG, col = idx % NG;
    const int g = col / HP, j = col % HP, kk = k % HP;
    float v = 0.f;
    if (kk < H && j < H) v = (k < HP ? p.Ru[d] : p.Rv[d])[(size_t)kk * 5 * H + g * H + j];
    Rs[k * LDR + col] = v;
  }
  for (int idx = tid; idx < 2 * (kRows + 1) * LDH; idx += 256) { hb[idx] = 0.f; cb[idx] = 0.f; }
  __syncthreads();

  float* zgd = p.zg[d];
  float* cd = p.c[d];
  float* hcd = p.hc[d];
  const int nsteps = wn > 0 ? Hh + wn - 1 : 0;

  // input part of the lane's (row, unit) pairs on diagonal s
  float zr[4][HT][5];
  auto prefetch = [&](int s) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = 16 * wave + 4 * lq + i, q = s - r;
      const bool on = r < Hh && q >= 0 && q < wn && s < nsteps;
      const size_t pix = on ? md_pixel(p, du, dv, wn, n, r, q) : 0;
#pragma unroll
      for (int t = 0; t < HT; ++t) {
        const int j = 16 * t + l16;
#pragma unroll
        for (int g = 0; g < 5; ++g) zr[i][t][g] = (on && j < H) ? zgd[pix * 5 * H + g * H + j] : 0.f;
      }
    }
  };
  prefetch(0);

  for (int s = 0; s < nsteps; ++s) {
    const float* hprev = hb + ((s + 1) & 1) * (kRows + 1) * LDH;
    const float* cprev = cb + ((s + 1) & 1) * (kRows + 1) * LDH;
    float* hcur = hb + (s & 1) * (kRows + 1) * LDH;
    float* ccur = cb + (s & 1) * (kRows + 1) * LDH;

    floatx4 acc[NTL];
#pragma unroll
    for (int nt = 0; nt < NTL; ++nt) acc[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
    // A[m][k]: m = row 16*wave + l16; k < HP: h of the row above (entry index = row), else h of the same row (index row + 1)
    const float* arow = hprev + (16 * wave + l16) * LDH;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int k = 4 * ks + lq;
      const float a = k < HP ? arow[k] : arow[LDH + k - HP];
#pragma unroll
      for (int nt = 0; nt < NTL; ++nt)
        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, Rs[k * LDR + nt * 16 + l16], acc[nt], 0, 0, 0);
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = 16 * wave + 4 * lq + i, q = s - r;
      const bool on = r < Hh && q >= 0 && q < wn;
      const size_t pix = on ? md_pixel(p, du, dv, wn, n, r, q) : 0;
#pragma unroll
      for (int t = 0; t < HT; ++t) {
        const int j = 16 * t + l16;
        const bool ok = on && j < H;
        const float gi = md_sigmoid(acc[0 * HT + t][i] + zr[i][t][0]);
        const float gfu = md_sigmoid(acc[1 * HT + t][i] + zr[i][t][1]);
        const float gfv = md_sigmoid(acc[2 * HT + t][i] + zr[i][t][2]);
        const float go = md_sigmoid(acc[3 * HT + t][i] + zr[i][t][3]);
        const float gg = md_tanh(acc[4 * HT + t][i] + zr[i][t][4]);
        const float h_up = hprev[r * LDH + j], h_left = hprev[(r + 1) * LDH + j];
        const float c_up = cprev[r * LDH + j], c_left = cprev[(r + 1) * LDH + j];
        const float ct = gfu * c_up + gfv * c_left + gi * gg;
        const float ht = go * md_tanh(ct);
        hcur[(r + 1) * LDH + j] = ok ? ht : 0.f;
        ccur[(r + 1) * LDH + j] = ok ? ct : 0.f;
        if (ok) {
          float* zrow = zgd + pix * 5 * H + j;
          zrow[0] = gi; zrow[H] = gfu; zrow[2 * H] = gfv; zrow[3 * H] = go; zrow[4 * H] = gg;
          cd[pix * H + j] = ct;
          p.y[pix * 4 * H + d * H + j] = ht;
          hcd[pix * 2 * H + j] = h_up;
          hcd[pix * 2 * H + H + j] = h_left;
        }
      }
    }
    prefetch(s + 1);
    __syncthreads();
  }

  // pixels beyond the image's width: y = 0, and zeros where the products after the backward pass read
  const int npad = (p.Ww - wn) * Hh;
  for (int idx = tid; idx < npad * H; idx += 256) {
    const int j = idx % H, cell = idx / H;
    const int u = cell / (p.Ww - wn), v = wn + cell % (p.Ww - wn);
    const size_t pix = ((size_t)u * p.Ww + v) * p.B + n;
    p.y[pix * 4 * H + d * H + j] = 0.f;
    cd[pix * H + j] = 0.f;
    hcd[pix * 2 * H + j] = 0.f;
    hcd[pix * 2 * H + H + j] = 0.f;
  }
}

template <int HT>
__global__ __launch_bounds__(256) void mdlstm_bwd_kernel(MdParams p) {
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
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
  const int wn = min(max(p.widths[n], 0), p.Ww);

  for (int idx = tid; idx < 2 * NG * HP; idx += 256) {
    const int k = idx / HP, j = idx % HP;
    const int kk = k % NG, g = kk / HP, jj = kk % HP;
    float v = 0.f;
    if (jj < H && j < H) v = (k < NG ? p.Ru[d] : p.Rv[d])[(size_t)j * 5 * H + g * H + jj];
    RT[k * LDT + j] = v;
  }
  for (int idx = tid; idx < (kRows + 1) * LDZ; idx += 256) dzb[idx] = 0.f;
  for (int idx = tid; idx < 2 * (kRows + 1) * LDH; idx += 256) { dcu[idx] = 0.f; dcv[idx] = 0.f; }
  __syncthreads();

  float* zgd = p.zg[d];
  const float* cd = p.c[d];
  const int nsteps = wn > 0 ? Hh + wn - 1 : 0;

  // gates, c, c of the two predecessors and dy of the lane's pairs on diagonal s
  float in[4][HT][9];
  auto prefetch = [&](int s) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = 16 * wave + 4 * lq + i, q = s - r;
      const bool on = s >= 0 && r < Hh && q >= 0 && q < wn;
      const size_t pix = on ? md_pixel(p, du, dv, wn, n, r, q) : 0;
      const size_t pup = (on && r >= 1) ? md_pixel(p, du, dv, wn, n, r - 1, q) : 0;
      const size_t plf = (on && q >= 1) ? md_pixel(p, du, dv, wn, n, r, q - 1) : 0;
#pragma unroll
      for (int t = 0; t < HT; ++t) {
        const int j = 16 * t + l16;
        const bool ok = on && j < H;
#pragma unroll
        for (int g = 0; g < 5; ++g) in[i][t][g] = ok ? zgd[pix * 5 * H + g * H + j] : 0.f;
        in[i][t][5] = ok ? cd[pix * H + j] : 0.f;
        in[i][t][6] = (ok && r >= 1) ? cd[pup * H + j] : 0.f;
        in[i][t][7] = (ok && q >= 1) ? cd[plf * H + j] : 0.f;
        in[i][t][8] = ok ? p.dy[pix * 4 * H + d * H + j] : 0.f;
      }
    }
  };
  prefetch(nsteps - 1);

  for (int s = nsteps - 1; s >= 0; --s) {
    const float* dcu_prev = dcu + ((s + 1) & 1) * (kRows + 1) * LDH;
    const float* dcv_prev = dcv + ((s + 1) & 1) * (kRows + 1) * LDH;
    float* dcu_cur = dcu + (s & 1) * (kRows + 1) * LDH;
    float* dcv_cur = dcv + (s & 1) * (kRows + 1) * LDH;

    // d h of diagonal s from d a of diagonal s+1: the successor below sits in row r+1, the one to the right in row r
    floatx4 acc[HT];
#pragma unroll
    for (int t = 0; t < HT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    const float* arow = dzb + (16 * wave + l16) * LDZ;
#pragma unroll 8
    for (int ks = 0; ks < KS; ++ks) {
      const int k = 4 * ks + lq;
      const float a = k < NG ? arow[LDZ + k] : arow[k - NG];
#pragma unroll
      for (int t = 0; t < HT; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, RT[k * LDT + t * 16 + l16], acc[t], 0, 0, 0);
    }
    __syncthreads();     // every wavefront has read the d a rows of diagonal s+1

#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = 16 * wave + 4 * lq + i, q = s - r;
      const bool on = r < Hh && q >= 0 && q < wn;
      const size_t pix = on ? md_pixel(p, du, dv, wn, n, r, q) : 0;
#pragma unroll
      for (int t = 0; t < HT; ++t) {
        const int j = 16 * t + l16;
        const bool ok = on && j < H;
        const float gi = in[i][t][0], gfu = in[i][t][1], gfv = in[i][t][2], go = in[i][t][3], gg = in[i][t][4];
        const float tc = md_tanh(in[i][t][5]);
        const float dh = in[i][t][8] + acc[t][i];
        const float d_o = dh * tc;
        const float dct = dcu_prev[(r + 1) * LDH + j] + dcv_prev[r * LDH + j] + dh * go * (1.0f - tc * tc);
        float dz[5];
        dz[0] = dct * gg * gi * (1.0f - gi);
        dz[1] = dct * in[i][t][6] * gfu * (1.0f - gfu);
        dz[2] = dct * in[i][t][7] * gfv * (1.0f - gfv);
        dz[3] = d_o * go * (1.0f - go);
        dz[4] = dct * gi * (1.0f - gg * gg);
        dcu_cur[r * LDH + j] = ok ? dct * gfu : 0.f;
        dcv_cur[r * LDH + j] = ok ? dct * gfv : 0.f;
#pragma unroll
        for (int g = 0; g < 5; ++g) dzb[r * LDZ + g * HP + j] = ok ? dz[g] : 0.f;
        if (ok) {
          float* zrow = zgd + pix * 5 * H + j;
#pragma unroll
          for (int g = 0; g < 5; ++g) zrow[g * H] = dz[g];
        }
      }
    }
    prefetch(s - 1);
    __syncthreads();
  }

  // d a = 0 beyond the image's width
  const int npad = (p.Ww - wn) * Hh;
  for (int idx = tid; idx < npad * 5 * H; idx += 256) {
    const int col = idx % (5 * H), cell = idx / (5 * H);
    const int u = cell / (p.Ww - wn), v = wn + cell % (p.Ww - wn);
    const size_t pix = ((size_t)u * p.Ww + v) * p.B + n;
    zgd[pix * 5 * H + col] = 0.f;
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
hipError_t md_launch(K kernel, int grid, size_t lds, hipStream_t stream, MdParams& p) {
  const void* fn = reinterpret_cast<const void*>(kernel);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  void* args[] = {&p};
  return hipLaunchKernel(fn, dim3((unsigned)grid), dim3(256), args, lds, stream);
}

MdParams md_params(const MdShape& s, const MdDir* dirs, const int32_t* widths) {
  MdParams p{};
  for (int d = 0; d < 4; ++d) {
    p.zg[d] = dirs[d].zg; p.c[d] = dirs[d].c; p.hc[d] = dirs[d].hc; p.Ru[d] = dirs[d].Ru; p.Rv[d] = dirs[d].Rv;
  }
  p.widths = widths; p.Hh = s.Hh; p.Ww = s.Ww; p.B = s.B; p.H = s.H;
  return p;
}

}  // namespace

bool mdlstm_supported(const MdShape& s) { return s.Hh >= 1 && s.Hh <= kRows && s.H >= 1 && s.H <= 32; }

hipError_t mdlstm_forward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths, float* y) {
  if (!mdlstm_supported(s)) return hipErrorInvalidValue;
  MdParams p = md_params(s, dirs, widths);
  p.y = y;
  if (s.H <= 16) return md_launch(mdlstm_fwd_kernel<1>, 4 * s.B, md_lds_fwd(1), stream, p);
  return md_launch(mdlstm_fwd_kernel<2>, 4 * s.B, md_lds_fwd(2), stream, p);
}

hipError_t mdlstm_backward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths, const float* dy) {
  if (!mdlstm_supported(s)) return hipErrorInvalidValue;
  MdParams p = md_params(s, dirs, widths);
  p.dy = dy;
  if (s.H <= 16) return md_launch(mdlstm_bwd_kernel<1>, 4 * s.B, md_lds_bwd(1), stream, p);
  return md_launch(mdlstm_bwd_kernel<2>, 4 * s.B, md_lds_bwd(2), stream, p);
}

}  // namespace rlstm
