// Stepwise engine of the recurrent part (Sec. 4.2 of the RETURNN paper): the same
// mathematics as the persistent kernels, written as one plain launch per time
// step with one thread per (sequence, unit).  It accepts any shape, uses the
// accurate libm sigmoid / tanh, and serves as the on-device cross-check of
// the persistent engine and as the path for shapes that do not fit on chip.
#include "rlstm_internal.h"

namespace rlstm {

namespace {

__device__ __forceinline__ float sigmoidf_(float u) { return 1.0f / (1.0f + expf(-u)); }

// ---------------------------------------------------------------------------
// stepwise engine: one launch per time step, one thread per (sequence, unit)
// ---------------------------------------------------------------------------
struct SFwdDir {
  float* zg; const float* R; const float* c0; float* y; float* c; float* hT; float* cT;
  float* hbuf;          // 2 x [B,H] carried h, double-buffered
  int direction;
};
struct SFwdParams { SFwdDir d[2]; const int32_t* seq_lens; int T, B, H, ldy, s, bf; };

__global__ __launch_bounds__(256) void step_fwd_kernel(SFwdParams p) {
  const SFwdDir& D = p.d[blockIdx.y];
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int B = p.B, H = p.H, T = p.T;
  if (j >= B * H) return;
  const int b = j / H, u = j % H;
  const int s = p.s;
  const int t = D.direction > 0 ? s : T - 1 - s;
  const int tprev = D.direction > 0 ? t - 1 : t + 1;
  const float* hprev = D.hbuf + (size_t)((s + 1) & 1) * B * H;
  float* hcur = D.hbuf + (size_t)(s & 1) * B * H;
  const size_t row = (size_t)t * B + b;
  float* zrow = D.zg + row * 4 * H + u;
  float a0 = zrow[0], a1 = zrow[H], a2 = zrow[2 * H], a3 = zrow[3 * H];
  for (int k = 0; k < H; ++k) {
    float hv = hprev[(size_t)b * H + k];
    const float* rr = D.R + (size_t)k * 4 * H + u;
    float r0 = rr[0], r1 = rr[H], r2 = rr[2 * H], r3 = rr[3 * H];
    if (p.bf) {   // bf16-operand variant: both factors rounded to bf16, fp32 accumulation
      hv = (float)(__bf16)hv;
      r0 = (float)(__bf16)r0; r1 = (float)(__bf16)r1; r2 = (float)(__bf16)r2; r3 = (float)(__bf16)r3;
    }
    a0 = fmaf(hv, r0, a0); a1 = fmaf(hv, r1, a1); a2 = fmaf(hv, r2, a2); a3 = fmaf(hv, r3, a3);
  }
  float cprev;
  if (tprev >= 0 && tprev < T) cprev = D.c[((size_t)tprev * B + b) * H + u];
  else cprev = D.c0 ? D.c0[(size_t)b * H + u] : 0.f;
  const float gi = sigmoidf_(a0), gf = sigmoidf_(a1), go = sigmoidf_(a2), gg = tanhf(a3);
  const float cn = gf * cprev + gi * gg;
  const float hn = go * tanhf(cn);
  const int len = min(max(p.seq_lens[b], 0), T);
  const bool valid = t < len;
  const float cs = valid ? cn : cprev;
  const float hs = valid ? hn : hprev[(size_t)b * H + u];
  zrow[0] = gi; zrow[H] = gf; zrow[2 * H] = go; zrow[3 * H] = gg;
  D.y[row * p.ldy + u] = valid ? hn : 0.f;
  D.c[row * H + u] = cs;
  hcur[(size_t)b * H + u] = hs;
  if (s == T - 1) {
    if (D.hT) D.hT[(size_t)b * H + u] = hs;
    if (D.cT) D.cT[(size_t)b * H + u] = cs;
  }
}

struct SInitParams { float* dst[2]; const float* src[2]; int ndir; size_t n; size_t off; };
// dst[d][off + i] = src[d] ? src[d][i] : 0
__global__ __launch_bounds__(256) void init_state_kernel(SInitParams p) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= p.n) return;
  for (int d = 0; d < p.ndir; ++d) p.dst[d][p.off + i] = p.src[d] ? p.src[d][i] : 0.f;
}

struct SBwdDir {
  float* zg; const float* R; const float* c; const float* c0; const float* dy;
  float* dh0; float* dc0;
  float* dhbuf;         // 2 x [B,H] carried Dh, double-buffered
  float* dcbuf;         // [B,H] carried Dc
  int direction;
};
struct SBwdParams { SBwdDir d[2]; const int32_t* seq_lens; int T, B, H, ldy, s, bf; };

// gate derivatives of step s: reads Dh of buffer (s+1)&1, writes dz in place and updates Dc
__global__ __launch_bounds__(256) void step_bwd_gates_kernel(SBwdParams p) {
  const SBwdDir& D = p.d[blockIdx.y];
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int B = p.B, H = p.H, T = p.T;
  if (j >= B * H) return;
  const int b = j / H, u = j % H;
  const int s = p.s;
  const int t = D.direction > 0 ? T - 1 - s : s;
  const int tprev = D.direction > 0 ? t - 1 : t + 1;
  const float Dh = D.dhbuf[(size_t)((s + 1) & 1) * B * H + j];
  const size_t row = (size_t)t * B + b;
  float* zrow = D.zg + row * 4 * H + u;
  const float gi = zrow[0], gf = zrow[H], go = zrow[2 * H], gg = zrow[3 * H];
  const float ct = D.c[row * H + u];
  float cp;
  if (tprev >= 0 && tprev < T) cp = D.c[((size_t)tprev * B + b) * H + u];
  else cp = D.c0 ? D.c0[(size_t)b * H + u] : 0.f;
  const int len = min(max(p.seq_lens[b], 0), T);
  float dz0 = 0.f, dz1 = 0.f, dz2 = 0.f, dz3 = 0.f;
  if (t < len) {
    const float tc = tanhf(ct);
    const float dh = D.dy[row * p.ldy + u] + Dh;
    const float d_o = dh * tc;
    const float dc = D.dcbuf[j] + dh * go * (1.0f - tc * tc);
    dz0 = dc * gg * gi * (1.0f - gi);
    dz1 = dc * cp * gf * (1.0f - gf);
    dz2 = d_o * go * (1.0f - go);
    dz3 = dc * gi * (1.0f - gg * gg);
    D.dcbuf[j] = dc * gf;
  }
  zrow[0] = dz0; zrow[H] = dz1; zrow[2 * H] = dz2; zrow[3 * H] = dz3;
  if (s == T - 1 && D.dc0) D.dc0[j] = D.dcbuf[j];
}

// Dh of buffer s&1 = dz_t R^T (+ Dh of buffer (s+1)&1 where the frame was invalid)
__global__ __launch_bounds__(256) void step_bwd_dh_kernel(SBwdParams p) {
  const SBwdDir& D = p.d[blockIdx.y];
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int B = p.B, H = p.H, T = p.T;
  if (j >= B * H) return;
  const int b = j / H, u = j % H;
  const int s = p.s;
  const int t = D.direction > 0 ? T - 1 - s : s;
  const float* dz = D.zg + ((size_t)t * B + b) * 4 * H;
  const float* rr = D.R + (size_t)u * 4 * H;
  float sum = 0.f;
  for (int k = 0; k < 4 * H; ++k) {
    float a = dz[k], r = rr[k];
    if (p.bf) { a = (float)(__bf16)a; r = (float)(__bf16)r; }
    sum = fmaf(a, r, sum);
  }
  const int len = min(max(p.seq_lens[b], 0), T);
  if (!(t < len)) sum += D.dhbuf[(size_t)((s + 1) & 1) * B * H + j];
  D.dhbuf[(size_t)(s & 1) * B * H + j] = sum;
  if (s == T - 1 && D.dh0) D.dh0[j] = sum;
}

__global__ __launch_bounds__(256) void column_sum_kernel(const float* __restrict__ a, size_t rows, int cols, int lda,
                                                          float* __restrict__ out) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= cols) return;
  float s = 0.f;
  for (size_t r = 0; r < rows; ++r) s += a[r * lda + n];
  out[n] = s;
}

// dR[k][n] += sum_b h0[b][k] * dz[tfirst(b)][b][n], tfirst = first processed valid frame
__global__ __launch_bounds__(256) void add_h0_outer_kernel(int T, int B, int H, int direction, const float* __restrict__ h0,
                                                            const float* __restrict__ dz, const int32_t* __restrict__ seq_lens,
                                                            float* __restrict__ dR) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)H * 4 * H) return;
  const int k = (int)(idx / (4 * H)), n = (int)(idx % (4 * H));
  float s = 0.f;
  for (int b = 0; b < B; ++b) {
    const int len = min(max(seq_lens[b], 0), T);
    if (len == 0) continue;
    const int tf = direction > 0 ? 0 : len - 1;
    s = fmaf(h0[(size_t)b * H + k], dz[((size_t)tf * B + b) * 4 * H + n], s);
  }
  dR[idx] += s;
}

__global__ void clear_flag_kernel(unsigned* flag) { *flag = 0u; }

__global__ __launch_bounds__(256) void copy_f32_kernel(float* __restrict__ dst, const float* __restrict__ src, size_t n) {
  const size_t n4 = n / 4;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride)
    reinterpret_cast<float4*>(dst)[i] = reinterpret_cast<const float4*>(src)[i];
  for (size_t i = n4 * 4 + (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}


}  // namespace

hipError_t device_info(DeviceInfo* out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  int cus = 0, lds = 0;
  e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
  if (e != hipSuccess) return e;
  out->num_cus = cus;
  out->max_lds = (size_t)lds;
  return hipSuccess;
}

hipError_t copy_f32(hipStream_t stream, float* dst, const float* src, size_t n) {
  hipLaunchKernelGGL(copy_f32_kernel, dim3(4096), dim3(256), 0, stream, dst, src, n);
  return hipGetLastError();
}

hipError_t clear_flag(hipStream_t stream, unsigned* flag) {
  hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, stream, flag);
  return hipGetLastError();
}

hipError_t column_sum(hipStream_t stream, const float* a, size_t rows, int cols, int lda, float* out) {
  hipLaunchKernelGGL(column_sum_kernel, dim3((unsigned)((cols + 255) / 256)), dim3(256), 0, stream, a, rows, cols, lda, out);
  return hipGetLastError();
}

hipError_t add_h0_outer(hipStream_t stream, int T, int B, int H, int direction, const float* h0,
                        const float* dz, const int32_t* seq_lens, float* dR) {
  const size_t total = (size_t)H * 4 * H;
  hipLaunchKernelGGL(add_h0_outer_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                     T, B, H, direction, h0, dz, seq_lens, dR);
  return hipGetLastError();
}

size_t stepwise_scratch_floats_per_dir(const RecShape& s) { return 3 * (size_t)s.B * s.H; }

// buf[d]: 2 x [B,H] carried h (double-buffered)
hipError_t stepwise_forward(hipStream_t stream, const RecShape& s, const RecFwdDir* dirs, const int32_t* seq_lens,
                            float* const* buf) {
  const size_t bh = (size_t)s.B * s.H;
  SInitParams ip{};
  SFwdParams kp{};
  for (int d = 0; d < s.ndir; ++d) {
    ip.dst[d] = buf[d]; ip.src[d] = dirs[d].h0;
    SFwdDir& k = kp.d[d];
    k.zg = dirs[d].zg; k.R = dirs[d].R; k.c0 = dirs[d].c0; k.y = dirs[d].y; k.c = dirs[d].c;
    k.hT = dirs[d].hT; k.cT = dirs[d].cT; k.hbuf = buf[d]; k.direction = dirs[d].direction;
  }
  ip.ndir = s.ndir; ip.n = bh; ip.off = bh;      // step 0 reads buffer 1
  kp.seq_lens = seq_lens; kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy; kp.bf = s.operand_dtype == 1 ? 1 : 0;
  const unsigned blocks = (unsigned)((bh + 255) / 256);
  hipLaunchKernelGGL(init_state_kernel, dim3(blocks), dim3(256), 0, stream, ip);
  for (int st = 0; st < s.T; ++st) {
    kp.s = st;
    hipLaunchKernelGGL(step_fwd_kernel, dim3(blocks, (unsigned)s.ndir), dim3(256), 0, stream, kp);
  }
  return hipGetLastError();
}

// buf[d]: [Dh buffer 0 | Dh buffer 1 | Dc], each [B,H]
hipError_t stepwise_backward(hipStream_t stream, const RecShape& s, const RecBwdDir* dirs, const int32_t* seq_lens,
                             float* const* buf) {
  const size_t bh = (size_t)s.B * s.H;
  SInitParams ih{}, ic{};
  SBwdParams kp{};
  for (int d = 0; d < s.ndir; ++d) {
    ih.dst[d] = buf[d]; ih.src[d] = dirs[d].dhT;
    ic.dst[d] = buf[d]; ic.src[d] = dirs[d].dcT;
    SBwdDir& k = kp.d[d];
    k.zg = dirs[d].zg; k.R = dirs[d].R; k.c = dirs[d].c; k.c0 = dirs[d].c0; k.dy = dirs[d].dy;
    k.dh0 = dirs[d].dh0; k.dc0 = dirs[d].dc0;
    k.dhbuf = buf[d]; k.dcbuf = buf[d] + 2 * bh; k.direction = dirs[d].direction;
  }
  ih.ndir = ic.ndir = s.ndir; ih.n = ic.n = bh; ih.off = bh; ic.off = 2 * bh;
  kp.seq_lens = seq_lens; kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy; kp.bf = s.operand_dtype == 1 ? 1 : 0;
  const unsigned blocks = (unsigned)((bh + 255) / 256);
  hipLaunchKernelGGL(init_state_kernel, dim3(blocks), dim3(256), 0, stream, ih);
  hipLaunchKernelGGL(init_state_kernel, dim3(blocks), dim3(256), 0, stream, ic);
  for (int st = 0; st < s.T; ++st) {
    kp.s = st;
    hipLaunchKernelGGL(step_bwd_gates_kernel, dim3(blocks, (unsigned)s.ndir), dim3(256), 0, stream, kp);
    hipLaunchKernelGGL(step_bwd_dh_kernel, dim3(blocks, (unsigned)s.ndir), dim3(256), 0, stream, kp);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  for (int d = 0; d < s.ndir; ++d) {
    e = column_sum(stream, dirs[d].zg, (size_t)s.T * s.B, 4 * s.H, 4 * s.H, dirs[d].db);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace rlstm
