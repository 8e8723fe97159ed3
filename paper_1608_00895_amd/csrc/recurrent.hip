// Dispatch of the recurrent passes to the persistent or the stepwise engine,
// and the layout of their scratch inside the caller's workspace.
#include "rlstm_internal.h"

namespace rlstm {

namespace {
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

size_t per_dir_bytes(const RecShape& s) {
  const size_t a = persistent_scratch_bytes_per_dir(s);
  const size_t b = stepwise_scratch_floats_per_dir(s) * sizeof(float);
  return align_up(a > b ? a : b, 256);
}
}  // namespace

size_t rec_workspace_bytes(const RecShape& s) { return 2 * per_dir_bytes(s); }

bool rec_persistent_supported(const RecShape& s, int num_cus, size_t max_lds) {
  return persistent_supported(s, num_cus, max_lds);
}

hipError_t rec_forward(hipStream_t stream, const RecShape& s, const RecFwdDir* dirs, const int32_t* seq_lens,
                       void* ws, unsigned* flag, bool persistent, int* resident_err) {
  char* base = static_cast<char*>(ws);
  char* scratch[2] = {base, base + per_dir_bytes(s)};
  if (persistent) return persistent_forward(stream, s, dirs, seq_lens, scratch, flag, resident_err);
  float* buf[2] = {reinterpret_cast<float*>(scratch[0]), reinterpret_cast<float*>(scratch[1])};
  return stepwise_forward(stream, s, dirs, seq_lens, buf);
}

hipError_t rec_backward(hipStream_t stream, const RecShape& s, const RecBwdDir* dirs, const int32_t* seq_lens,
                        void* ws, unsigned* flag, bool persistent, int* resident_err) {
  char* base = static_cast<char*>(ws);
  char* scratch[2] = {base, base + per_dir_bytes(s)};
  if (persistent) return persistent_backward(stream, s, dirs, seq_lens, scratch, flag, resident_err);
  float* buf[2] = {reinterpret_cast<float*>(scratch[0]), reinterpret_cast<float*>(scratch[1])};
  return stepwise_backward(stream, s, dirs, seq_lens, buf);
}

}  // namespace rlstm
