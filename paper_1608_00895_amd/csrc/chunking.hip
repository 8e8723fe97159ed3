// Chunking (Sec. 4 of the RETURNN paper): sequences of very different lengths are cut into
// segments of constant length, possibly overlapping, so that a minibatch of segments carries
// little zero padding; the experiments (Sec. 6) use segments of 250 frames, zero-padded where
// a sequence ends, 81 segments per batch.
//
// A segment table (host, integer work only) and a gather kernel that builds the time-major
// minibatch of segments on the device.
#include "rlstm_internal.h"

namespace rlstm {

// Segments of a sequence of n frames start at frames 0, step, 2*step, ... (every start < n) and
// hold min(size, n - start) frames.  Table order: sequence by sequence, starts ascending.
long long chunk_plan(const int32_t* seq_lens, int B, int size, int step, int32_t* seq, int32_t* start, int32_t* len,
                     long long max_chunks) {
  long long k = 0;
  for (int b = 0; b < B; ++b) {
    const int n = seq_lens[b];
    for (int t = 0; t < n; t += step) {
      if (k < max_chunks) {
        if (seq) seq[k] = b;
        if (start) start[k] = t;
        if (len) len[k] = n - t < size ? n - t : size;
      }
      ++k;
    }
  }
  return k;
}

namespace {
struct GatherParams {
  const float* x; float* xc;
  const int32_t* seq; const int32_t* start; const int32_t* len;
  int T, B, D, ldx, size, nchunks;
};
// one thread per element of xc [size, nchunks, D]
__global__ __launch_bounds__(256) void chunk_gather_kernel(GatherParams p) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t total = (size_t)p.size * p.nchunks * p.D;
  if (idx >= total) return;
  const int i = (int)(idx % p.D);
  const int k = (int)((idx / p.D) % p.nchunks);
  const int t = (int)(idx / ((size_t)p.D * p.nchunks));
  const int b = p.seq[k], t0 = p.start[k], n = p.len[k];
  float v = 0.f;
  // a table entry that points outside x is treated as padding rather than read
  if (t < n && b >= 0 && b < p.B && t0 >= 0 && t0 + t < p.T) v = p.x[((size_t)(t0 + t) * p.B + b) * p.ldx + i];
  p.xc[idx] = v;
}
}  // namespace

hipError_t chunk_gather(hipStream_t stream, const float* x, int T, int B, int D, int ldx, const int32_t* seq,
                        const int32_t* start, const int32_t* len, int nchunks, int size, float* xc) {
  GatherParams p{x, xc, seq, start, len, T, B, D, ldx, size, nchunks};
  const size_t total = (size_t)size * nchunks * D;
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL(chunk_gather_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace rlstm
