// Helpers of the streaming mode: a unidirectional LSTM stack reads its sequences segment by segment, every
// segment starting from the final state of the one before (Sec. 3.2: final states passed on from one
// recurrent layer to another; Sec. 4: cutting into segments otherwise gives up the context in the end
// states).  The layer kernels are those of the one-segment path; here are only the per-segment length
// table, the accumulation of the bias gradients over the segments and a fill.
#include "rlstm_internal.h"

namespace rlstm {

namespace {

// out[s * B + b] = clamp(seq_lens[b] - s * Tc, 0, Tc): valid frames of sequence b inside segment s
__global__ __launch_bounds__(256) void segment_lens_kernel(const int32_t* __restrict__ seq_lens, int B, int S, int Tc,
                                                           int32_t* __restrict__ out) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= S * B) return;
  const int s = i / B, b = i % B;
  const long long left = (long long)seq_lens[b] - (long long)s * Tc;
  out[i] = (int32_t)(left < 0 ? 0 : (left > Tc ? Tc : left));
}

// dst = src (assign) or dst += src
__global__ __launch_bounds__(256) void accumulate_kernel(float* __restrict__ dst, const float* __restrict__ src, size_t n,
                                                         int assign) {
  const size_t gsz = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += gsz) dst[i] = assign ? src[i] : dst[i] + src[i];
}

__global__ __launch_bounds__(256) void fill_kernel(float* __restrict__ dst, size_t n, float v) {
  const size_t gsz = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += gsz) dst[i] = v;
}

inline unsigned grid_for(size_t n) {
  const size_t g = (n + 255) / 256;
  return (unsigned)(g > 2048 ? 2048 : (g ? g : 1));
}

}  // namespace

hipError_t segment_lens(hipStream_t stream, const int32_t* seq_lens, int B, int S, int Tc, int32_t* out) {
  hipLaunchKernelGGL(segment_lens_kernel, dim3((unsigned)(((size_t)S * B + 255) / 256)), dim3(256), 0, stream, seq_lens, B, S,
                     Tc, out);
  return hipGetLastError();
}

hipError_t accumulate(hipStream_t stream, float* dst, const float* src, size_t n, bool assign) {
  hipLaunchKernelGGL(accumulate_kernel, dim3(grid_for(n)), dim3(256), 0, stream, dst, src, n, assign ? 1 : 0);
  return hipGetLastError();
}

hipError_t fill_f32(hipStream_t stream, float* dst, size_t n, float v) {
  hipLaunchKernelGGL(fill_kernel, dim3(grid_for(n)), dim3(256), 0, stream, dst, n, v);
  return hipGetLastError();
}

}  // namespace rlstm
