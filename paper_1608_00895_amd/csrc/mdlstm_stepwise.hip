// Stepwise engine of the two-dimensional LSTM layer (Sec. 4.2 of the RETURNN paper: the state of pixel (u, v)
// depends on its two predecessors in scan order, so all pixels of an anti-diagonal can be computed together):
// ONE LAUNCH PER ANTI-DIAGONAL, plain kernels, one thread per (scan direction, pixel of the diagonal, image, unit).
// It takes every shape (any height, any number of units) and is the engine for shapes the scan kernels of
// mdlstm.hip cannot hold; it is also the on-device cross-check of those kernels.  Same buffers and layouts as the
// scan kernels (rlstm_internal.h): zg [P, 5H] (b + x W in, activated gates out, d loss / d a after the backward
// pass), c [P, H], hc [P, S] = [h_up | h_left | ...], y / dy [P, 4H].
//
// The anti-diagonals are those of the PADDED array (all Ww columns): a pixel at or beyond its image's width gets
// h = c = y = 0, which is exactly the zero state a predecessor outside the image contributes, so every image
// computes as if alone, also in the directions that start at the padded side.
#include "rlstm_internal.h"

#include <cmath>

namespace rlstm {

namespace {

struct MdStepParams {
  float* zg[4]; float* c[4]; float* hc[4];
  const float* Ru[4]; const float* Rv[4];
  float* dcu[4]; float* dcv[4];       // backward scratch [P, H]: d c~ * f_u and d c~ * f_v of every pixel
  float* y; const float* dy;
  const int32_t* widths;
  int Hh, Ww, B, H, S;
  int diag, r0, nr;                   // anti-diagonal, its first row (scan coordinates) and number of rows
};

__device__ __forceinline__ float sigmoidf_(float u) { return 1.0f / (1.0f + expf(-u)); }

// scan coordinates (u', v') of direction d -> image coordinates
__device__ __forceinline__ void md_coords(const MdStepParams& p, int d, int us, int vs, int& u, int& v, int& du, int& dv) {
  du = (d & 2) ? -1 : 1;
  dv = (d & 1) ? -1 : 1;
  u = du > 0 ? us : p.Hh - 1 - us;
  v = dv > 0 ? vs : p.Ww - 1 - vs;
}

__global__ __launch_bounds__(256) void mdlstm_step_fwd_kernel(MdStepParams p) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int H = p.H;
  if (idx >= (size_t)4 * p.nr * p.B * H) return;
  const int j = (int)(idx % H);
  const int n = (int)((idx / H) % p.B);
  const int r = (int)((idx / ((size_t)H * p.B)) % p.nr);
  const int d = (int)(idx / ((size_t)H * p.B * p.nr));
  int u, v, du, dv;
  md_coords(p, d, p.r0 + r, p.diag - (p.r0 + r), u, v, du, dv);
  const int wn = min(max(p.widths[n], 0), p.Ww);
  const bool inside = v < wn;
  const size_t pix = ((size_t)u * p.Ww + v) * p.B + n;
  const int pu = u - du, pv = v - dv;
  const bool has_up = pu >= 0 && pu < p.Hh, has_left = pv >= 0 && pv < p.Ww;
  const size_t pix_up = ((size_t)(has_up ? pu : u) * p.Ww + v) * p.B + n;
  const size_t pix_left = ((size_t)u * p.Ww + (has_left ? pv : v)) * p.B + n;
  const float* hup = p.y + pix_up * 4 * H + (size_t)d * H;      // y holds h, zero outside the images
  const float* hleft = p.y + pix_left * 4 * H + (size_t)d * H;
  float a[5];
#pragma unroll
  for (int g = 0; g < 5; ++g) a[g] = p.zg[d][pix * 5 * H + g * H + j];
  if (has_up) {
    for (int k = 0; k < H; ++k) {
      const float h = hup[k];
      const float* row = p.Ru[d] + (size_t)k * 5 * H + j;
#pragma unroll
      for (int g = 0; g < 5; ++g) a[g] += h * row[g * H];
    }
  }
  if (has_left) {
    for (int k = 0; k < H; ++k) {
      const float h = hleft[k];
      const float* row = p.Rv[d] + (size_t)k * 5 * H + j;
#pragma unroll
      for (int g = 0; g < 5; ++g) a[g] += h * row[g * H];
    }
  }
  const float gi = sigmoidf_(a[0]), gfu = sigmoidf_(a[1]), gfv = sigmoidf_(a[2]), go = sigmoidf_(a[3]), gg = tanhf(a[4]);
  const float c_up = has_up ? p.c[d][pix_up * H + j] : 0.f;
  const float c_left = has_left ? p.c[d][pix_left * H + j] : 0.f;
  const float ct = gfu * c_up + gfv * c_left + gi * gg;
  const float ht = go * tanhf(ct);
  float* zrow = p.zg[d] + pix * 5 * H + j;
  zrow[0] = gi; zrow[H] = gfu; zrow[2 * H] = gfv; zrow[3 * H] = go; zrow[4 * H] = gg;
  p.c[d][pix * H + j] = inside ? ct : 0.f;
  p.y[pix * 4 * H + (size_t)d * H + j] = inside ? ht : 0.f;
  p.hc[d][pix * p.S + j] = has_up ? hup[j] : 0.f;
  p.hc[d][pix * p.S + H + j] = has_left ? hleft[j] : 0.f;
}

__global__ __launch_bounds__(256) void mdlstm_step_bwd_kernel(MdStepParams p) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int H = p.H;
  if (idx >= (size_t)4 * p.nr * p.B * H) return;
  const int j = (int)(idx % H);
  const int n = (int)((idx / H) % p.B);
  const int r = (int)((idx / ((size_t)H * p.B)) % p.nr);
  const int d = (int)(idx / ((size_t)H * p.B * p.nr));
  int u, v, du, dv;
  md_coords(p, d, p.r0 + r, p.diag - (p.r0 + r), u, v, du, dv);
  const int wn = min(max(p.widths[n], 0), p.Ww);
  const bool inside = v < wn;
  const size_t pix = ((size_t)u * p.Ww + v) * p.B + n;
  const int pu = u - du, pv = v - dv, su = u + du, sv = v + dv;
  const bool has_up = pu >= 0 && pu < p.Hh, has_left = pv >= 0 && pv < p.Ww;
  const bool has_su = su >= 0 && su < p.Hh, has_sv = sv >= 0 && sv < p.Ww;
  // gradient arriving from the two successors (computed by the launch before this one)
  float Dh = 0.f, Dc = 0.f;
  if (has_su) {
    const size_t q = ((size_t)su * p.Ww + v) * p.B + n;
    const float* dz = p.zg[d] + q * 5 * H;
    const float* row = p.Ru[d] + (size_t)j * 5 * H;
    float acc = 0.f;
    for (int k = 0; k < 5 * H; ++k) acc += dz[k] * row[k];
    Dh += acc;
    Dc += p.dcu[d][q * H + j];
  }
  if (has_sv) {
    const size_t q = ((size_t)u * p.Ww + sv) * p.B + n;
    const float* dz = p.zg[d] + q * 5 * H;
    const float* row = p.Rv[d] + (size_t)j * 5 * H;
    float acc = 0.f;
    for (int k = 0; k < 5 * H; ++k) acc += dz[k] * row[k];
    Dh += acc;
    Dc += p.dcv[d][q * H + j];
  }
  float* zrow = p.zg[d] + pix * 5 * H + j;
  float dz[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
  float dct = 0.f, gfu = 0.f, gfv = 0.f;
  if (inside) {
    const float gi = zrow[0], go = zrow[3 * H], gg = zrow[4 * H];
    gfu = zrow[H]; gfv = zrow[2 * H];
    const float c_up = has_up ? p.c[d][(((size_t)pu * p.Ww + v) * p.B + n) * H + j] : 0.f;
    const float c_left = has_left ? p.c[d][(((size_t)u * p.Ww + pv) * p.B + n) * H + j] : 0.f;
    const float tc = tanhf(p.c[d][pix * H + j]);
    const float dh = p.dy[pix * 4 * H + (size_t)d * H + j] + Dh;
    dct = Dc + dh * go * (1.0f - tc * tc);
    dz[0] = dct * gg * gi * (1.0f - gi);
    dz[1] = dct * c_up * gfu * (1.0f - gfu);
    dz[2] = dct * c_left * gfv * (1.0f - gfv);
    dz[3] = dh * tc * go * (1.0f - go);
    dz[4] = dct * gi * (1.0f - gg * gg);
  }
  // Every thread of the launch reads only its own unit's gates of this pixel and the d a of OTHER pixels (the
  // successors', written by the launch before): overwriting in place races with nobody.
#pragma unroll
  for (int g = 0; g < 5; ++g) zrow[g * H] = dz[g];
  p.dcu[d][pix * H + j] = dct * gfu;
  p.dcv[d][pix * H + j] = dct * gfv;
}

MdStepParams step_params(const MdShape& s, const MdDir* dirs, const int32_t* widths) {
  MdStepParams p{};
  for (int d = 0; d < 4; ++d) {
    p.zg[d] = dirs[d].zg; p.c[d] = dirs[d].c; p.hc[d] = dirs[d].hc; p.Ru[d] = dirs[d].Ru; p.Rv[d] = dirs[d].Rv;
  }
  p.widths = widths; p.Hh = s.Hh; p.Ww = s.Ww; p.B = s.B; p.H = s.H; p.S = s.S;
  return p;
}

// rows (scan coordinates) of anti-diagonal `diag` of an Hh x Ww array
inline void diag_rows(const MdShape& s, int diag, int& r0, int& nr) {
  r0 = diag - (s.Ww - 1) > 0 ? diag - (s.Ww - 1) : 0;
  const int r1 = diag < s.Hh - 1 ? diag : s.Hh - 1;
  nr = r1 - r0 + 1;
}

}  // namespace

size_t mdlstm_stepwise_scratch_floats(const MdShape& s) { return (size_t)8 * s.Hh * s.Ww * s.B * s.H; }

hipError_t mdlstm_stepwise_forward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths, float* y) {
  MdStepParams p = step_params(s, dirs, widths);
  p.y = y;
  for (int diag = 0; diag < s.Hh + s.Ww - 1; ++diag) {
    diag_rows(s, diag, p.r0, p.nr);
    p.diag = diag;
    const size_t items = (size_t)4 * p.nr * s.B * s.H;
    hipLaunchKernelGGL(mdlstm_step_fwd_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, stream, p);
  }
  return hipGetLastError();
}

hipError_t mdlstm_stepwise_backward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths,
                                    const float* dy, float* scratch, float* const* db) {
  MdStepParams p = step_params(s, dirs, widths);
  p.dy = dy;
  const size_t ph = (size_t)s.Hh * s.Ww * s.B * s.H;
  for (int d = 0; d < 4; ++d) { p.dcu[d] = scratch + (size_t)(2 * d) * ph; p.dcv[d] = scratch + (size_t)(2 * d + 1) * ph; }
  for (int diag = s.Hh + s.Ww - 2; diag >= 0; --diag) {
    diag_rows(s, diag, p.r0, p.nr);
    p.diag = diag;
    const size_t items = (size_t)4 * p.nr * s.B * s.H;
    hipLaunchKernelGGL(mdlstm_step_bwd_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, stream, p);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t P = (size_t)s.Hh * s.Ww * s.B;
  for (int d = 0; d < 4 && e == hipSuccess; ++d) e = column_sum(stream, dirs[d].zg, P, 5 * s.H, 5 * s.H, db[d]);
  return e;
}

}  // namespace rlstm
