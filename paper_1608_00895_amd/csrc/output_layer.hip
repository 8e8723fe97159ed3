// Frame-wise softmax / cross-entropy output layer on top of the stack and the parameter updates
// (Secs. 3.2, 4.3 and 6 of the RETURNN paper: cross-entropy output layer, 1501 classes per frame,
// frame error rate; SGD with momentum or Adam; batch gradients are sums; padded frames have no
// influence).  The affine map and its gradients are the MFMA products of gemm.hip; here are the
// row-wise softmax / loss / error kernel, the deterministic reductions and the update kernels.
#include "rlstm_internal.h"

#include <cmath>

namespace rlstm {

namespace {

// (value, index) with "larger value, then smaller index" order
struct Best { float v; int i; };
__device__ __forceinline__ Best better(Best a, Best b) { return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a; }

struct CeParams {
  float* z;                  // [rows, ld] logits in columns [0, C); d loss / d logits out, columns [C, ld) zeroed
  const int32_t* labels;     // [rows]
  const int32_t* seq_lens;   // [B]
  float* row_loss;           // [rows]
  int32_t* row_err;          // [rows]
  int T, B, C, ld;
};

// One workgroup per frame (t, b).  Frames outside their sequence, and frames whose label is not a
// class index, contribute nothing: zero row, zero loss, no error.
__global__ __launch_bounds__(256) void softmax_ce_rows_kernel(CeParams p) {
  __shared__ float sv[4];
  __shared__ int si[4];
  __shared__ float ssum[4];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = row / p.B, b = row % p.B;
  float* z = p.z + (size_t)row * p.ld;
  const int len = min(max(p.seq_lens[b], 0), p.T);
  const int label = p.labels[row];
  if (t >= len || label < 0 || label >= p.C) {
    for (int i = tid; i < p.ld; i += 256) z[i] = 0.f;
    if (tid == 0) { p.row_loss[row] = 0.f; p.row_err[row] = 0; }
    return;
  }
  // largest logit and its first index
  Best best{-INFINITY, 0x7fffffff};
  for (int i = tid; i < p.C; i += 256) best = better(best, Best{z[i], i});
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    Best o{__shfl_xor(best.v, off), __shfl_xor(best.i, off)};
    best = better(best, o);
  }
  if (lane == 0) { sv[wave] = best.v; si[wave] = best.i; }
  __syncthreads();
  best = Best{sv[0], si[0]};
#pragma unroll
  for (int w = 1; w < 4; ++w) best = better(best, Best{sv[w], si[w]});
  // sum of exp(z - max), fixed reduction tree
  float s = 0.f;
  for (int i = tid; i < p.C; i += 256) s += expf(z[i] - best.v);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
  if (lane == 0) ssum[wave] = s;
  __syncthreads();
  s = (ssum[0] + ssum[1]) + (ssum[2] + ssum[3]);
  const float lse = best.v + logf(s);
  const float zl = z[label];
  __syncthreads();           // every thread has read z[label] before the row is overwritten
  for (int i = tid; i < p.ld; i += 256) z[i] = i < p.C ? expf(z[i] - lse) - (i == label ? 1.f : 0.f) : 0.f;
  if (tid == 0) { p.row_loss[row] = lse - zl; p.row_err[row] = best.i != label ? 1 : 0; }
}

// loss = sum of row_loss, errors = sum of row_err: one workgroup, each thread a strided share, fixed tree
__global__ __launch_bounds__(1024) void ce_total_kernel(const float* row_loss, const int32_t* row_err, int rows,
                                                         float* loss, int32_t* errors) {
  __shared__ float sl[1024];
  __shared__ int se[1024];
  const int tid = threadIdx.x;
  float l = 0.f;
  int e = 0;
  for (int i = tid; i < rows; i += 1024) { l += row_loss[i]; e += row_err[i]; }
  sl[tid] = l; se[tid] = e;
  __syncthreads();
  for (int off = 512; off >= 1; off >>= 1) {
    if (tid < off) { sl[tid] += sl[tid + off]; se[tid] += se[tid + off]; }
    __syncthreads();
  }
  if (tid == 0) { *loss = sl[0]; *errors = se[0]; }
}

// column sums of a [rows, cols] matrix (row stride ld) in two deterministic stages: kChunks partial sums per column, then their sum
constexpr int kChunks = 128;
__global__ __launch_bounds__(256) void colsum_partial_kernel(const float* a, int rows, int cols, int ld, float* partial) {
  const int c = blockIdx.x * 256 + threadIdx.x, chunk = blockIdx.y;
  if (c >= cols) return;
  const int per = (rows + kChunks - 1) / kChunks;
  const int r0 = chunk * per, r1 = min(rows, r0 + per);
  float s = 0.f;
  for (int r = r0; r < r1; ++r) s += a[(size_t)r * ld + c];
  partial[(size_t)chunk * cols + c] = s;
}
__global__ __launch_bounds__(256) void colsum_final_kernel(const float* partial, int cols, float* out) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= cols) return;
  float s = 0.f;
  for (int k = 0; k < kChunks; ++k) s += partial[(size_t)k * cols + c];
  out[c] = s;
}

__global__ __launch_bounds__(256) void sgd_momentum_kernel(float* p, const float* g, float* v, size_t n, float lr, float mu) {
  const size_t gsz = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += gsz) {
    const float vel = mu * v[i] + g[i];
    v[i] = vel;
    p[i] -= lr * vel;
  }
}
__global__ __launch_bounds__(256) void adam_kernel(float* p, const float* g, float* m, float* v, size_t n, float lr,
                                                   float b1, float omb1, float b2, float omb2, float eps, float c1, float c2) {
  const size_t gsz = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += gsz) {
    const float gi = g[i];
    const float mi = b1 * m[i] + omb1 * gi;            // omb = 1 - b, rounded once from the double
    const float vi = b2 * v[i] + omb2 * gi * gi;
    m[i] = mi; v[i] = vi;
    p[i] -= lr * (mi * c1) / (sqrtf(vi * c2) + eps);   // c1 = 1 / (1 - b1^t), c2 = 1 / (1 - b2^t)
  }
}

// dst[r, 0..cols_dst) = src[r, 0..cols_src) followed by zeros (row strides ld_dst, ld_src)
__global__ __launch_bounds__(256) void repitch_kernel(const float* src, int ld_src, int cols_src, float* dst, int ld_dst,
                                                      int cols_dst, int rows) {
  const size_t total = (size_t)rows * cols_dst, gsz = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += gsz) {
    const int r = (int)(i / cols_dst), c = (int)(i % cols_dst);
    dst[(size_t)r * ld_dst + c] = c < cols_src ? src[(size_t)r * ld_src + c] : 0.f;
  }
}

inline unsigned grid_for(size_t n) {
  const size_t g = (n + 255) / 256;
  return (unsigned)(g > 4096 ? 4096 : (g ? g : 1));
}

}  // namespace

size_t ce_scratch_floats(int rows, int C) { return 2 * (size_t)rows + (size_t)kChunks * C; }

hipError_t repitch(hipStream_t stream, const float* src, int ld_src, int cols_src, float* dst, int ld_dst, int cols_dst, int rows) {
  hipLaunchKernelGGL(repitch_kernel, dim3(grid_for((size_t)rows * cols_dst)), dim3(256), 0, stream, src, ld_src, cols_src, dst,
                     ld_dst, cols_dst, rows);
  return hipGetLastError();
}

hipError_t softmax_ce_rows(hipStream_t stream, float* z, int ld, const int32_t* labels, const int32_t* seq_lens, int T, int B,
                           int C, float* scratch, float* loss, int32_t* errors, float* dbo) {
  const int rows = T * B;
  CeParams p{z, labels, seq_lens, scratch, reinterpret_cast<int32_t*>(scratch + rows), T, B, C, ld};
  hipLaunchKernelGGL(softmax_ce_rows_kernel, dim3((unsigned)rows), dim3(256), 0, stream, p);
  hipLaunchKernelGGL(ce_total_kernel, dim3(1), dim3(1024), 0, stream, p.row_loss, p.row_err, rows, loss, errors);
  float* partial = scratch + 2 * (size_t)rows;
  hipLaunchKernelGGL(colsum_partial_kernel, dim3((unsigned)((C + 255) / 256), kChunks), dim3(256), 0, stream, z, rows, C, ld, partial);
  hipLaunchKernelGGL(colsum_final_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, stream, partial, C, dbo);
  return hipGetLastError();
}

hipError_t sgd_momentum(hipStream_t stream, float* p, const float* g, float* v, size_t n, float lr, float mu) {
  hipLaunchKernelGGL(sgd_momentum_kernel, dim3(grid_for(n)), dim3(256), 0, stream, p, g, v, n, lr, mu);
  return hipGetLastError();
}

hipError_t adam(hipStream_t stream, float* p, const float* g, float* m, float* v, size_t n, double lr, double b1, double b2,
                double eps, int step) {
  const double c1 = 1.0 / (1.0 - pow(b1, step)), c2 = 1.0 / (1.0 - pow(b2, step));
  hipLaunchKernelGGL(adam_kernel, dim3(grid_for(n)), dim3(256), 0, stream, p, g, m, v, n, (float)lr, (float)b1,
                     (float)(1.0 - b1), (float)b2, (float)(1.0 - b2), (float)eps, (float)c1, (float)c2);
  return hipGetLastError();
}

}  // namespace rlstm
