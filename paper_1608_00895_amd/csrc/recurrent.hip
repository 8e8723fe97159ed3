// Dispatch of the recurrent passes to the persistent or the stepwise engine,
// and the layout of their scratch inside the caller's workspace.
#include "rlstm_internal.h"

namespace rlstm {

namespace {
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

size_t stepwise_dir_bytes(const RecShape& s) { return align_up(stepwise_scratch_floats_per_dir(s) * sizeof(float), 256); }
}  // namespace

size_t rec_workspace_bytes(const RecShape& s) {
  const size_t a = persistent_scratch_bytes(s), b = 2 * stepwise_dir_bytes(s);
  return align_up(a > b ? a : b, 256);
}

size_t rec_workspace_bytes_fwd(const RecShape& s) {
  const size_t a = persistent_scratch_bytes_fwd(s), b = 2 * stepwise_dir_bytes(s);
  return align_up(a > b ? a : b, 256);
}

bool rec_persistent_supported(const RecShape& s, int num_cus, size_t max_lds) {
  return persistent_supported(s, num_cus, max_lds);
}

hipError_t rec_forward(hipStream_t stream, const RecShape& s, const RecFwdDir* dirs, const int32_t* seq_lens,
                       void* ws, unsigned* flag, bool persistent, int* resident_err, int s_begin, int s_end) {
  char* base = static_cast<char*>(ws);
  if (persistent) return persistent_forward(stream, s, dirs, seq_lens, base, flag, resident_err, s_begin, s_end);
  if (s_begin != 0 || s_end != s.T) return hipErrorInvalidValue;
  float* buf[2] = {reinterpret_cast<float*>(base), reinterpret_cast<float*>(base + stepwise_dir_bytes(s))};
  return stepwise_forward(stream, s, dirs, seq_lens, buf);
}

hipError_t rec_backward(hipStream_t stream, const RecShape& s, const RecBwdDir* dirs, const int32_t* seq_lens,
                        void* ws, unsigned* flag, bool persistent, int* resident_err, int s_begin, int s_end) {
  char* base = static_cast<char*>(ws);
  if (persistent) return persistent_backward(stream, s, dirs, seq_lens, base, flag, resident_err, s_begin, s_end);
  if (s_begin != 0 || s_end != s.T) return hipErrorInvalidValue;
  float* buf[2] = {reinterpret_cast<float*>(base), reinterpret_cast<float*>(base + stepwise_dir_bytes(s))};
  return stepwise_backward(stream, s, dirs, seq_lens, buf);
}

}  // namespace rlstm
