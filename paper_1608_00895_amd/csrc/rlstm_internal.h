// Internal declarations shared by the translation units of librlstm.
// Nothing here is part of the C ABI (see include/rlstm.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace rlstm {

// ---------------------------------------------------------------------------
// Dense products on the matrix cores.
//   C[M,N] (row stride ldc) = op(A) * op(B) (+ bias[n]) (+ C if accumulate)
//   transA == false: A is [M,K], row stride lda (k contiguous)
//   transA == true : A is stored [K,M], row stride lda (m contiguous)
//   transB == false: B is [K,N], row stride ldb (n contiguous)
//   transB == true : B is stored [N,K], row stride ldb (k contiguous)
// splitk_ws / splitk_floats: scratch for deterministic split-K partial sums
// (may be null: no split).  naive selects the plain one-thread-per-output
// kernel of the stepwise engine.
// ---------------------------------------------------------------------------
constexpr int kVariantNoWalk = 13, kVariantNoRing = 14;
struct GemmCall {
  bool transA = false, transB = false;
  int M = 0, N = 0, K = 0;
  const float* A = nullptr; int lda = 0;
  const float* B = nullptr; int ldb = 0;
  float* C = nullptr; int ldc = 0;
  const float* bias = nullptr;
  bool accumulate = false;
  float* splitk_ws = nullptr; size_t splitk_floats = 0;
  int operand_dtype = 0;
  bool naive = false;
  bool small_footprint = false;   // runs beside the recurrent kernels on shared CUs: keep to the plain 128 x 128 kernel
  // fp32 operands: 0 the product from three bf16 parts per operand, 1 the pipelined fp32-instruction kernel wherever it
  // applies, 2 the plain fp32-instruction kernel, 3 the fp32-instruction kernels chosen by call (pipelined alone, the
  // short instruction beside the recurrent kernels); bf16 copies: kVariantNoWalk, kVariantNoRing (measurement)
  int variant = 0;
  // operand_dtype 1 only: bf16 copies of op(A) and op(B) (written by to_bf16 / to_bf16_2d), in a layout of their own:
  // transA16 == false: A16 is [M,K] with row stride lda16 (k contiguous); true: stored [K,M]; B16 likewise (transB16
  // == false: [K,N]; true: stored [N,K]).  They are used instead of A and B where the kernel that takes bf16 from
  // memory runs; A and B stay valid (other kernels read them).  require_mem16: fail with hipErrorInvalidValue
  // instead of falling back.
  const unsigned short* A16 = nullptr; const unsigned short* B16 = nullptr;
  int lda16 = 0, ldb16 = 0;
  bool transA16 = false, transB16 = false;
  bool require_mem16 = false;
};
hipError_t gemm(hipStream_t stream, const GemmCall& g);
// dst[i] = bf16(src[i]) (round to nearest even); n a multiple of 8, both arrays 16-byte aligned
hipError_t to_bf16(hipStream_t stream, const float* src, unsigned short* dst, size_t n);
// src [R, C] fp32 (row stride ld, a multiple of 4) -> dst [R, C] bf16 with row stride ldd (0: C; a multiple of 8; dst
// may be null) and its transpose dstT [C, R] bf16, dense (or null); R, C multiples of 8, all arrays 16-byte aligned
hipError_t to_bf16_2d(hipStream_t stream, const float* src, int R, int C, int ld, unsigned short* dst, int ldd, unsigned short* dstT);

// ---------------------------------------------------------------------------
// Recurrent passes.  One call handles ndir (1 or 2) independent directions of
// the same shape in a single launch.
// ---------------------------------------------------------------------------
struct RecFwdDir {
  float* zg;          // [T,B,4H] in: b + x W ; out: activated gates i|f|o|g
  const float* R;     // [H,4H]
  const float* h0;    // [B,H] or null
  const float* c0;    // [B,H] or null
  float* y;           // [T,B,ldy], already offset to this direction's columns
  float* c;           // [T,B,H]
  float* hT;          // [B,H] or null
  float* cT;          // [B,H] or null
  int direction;      // +1 / -1
};
struct RecBwdDir {
  float* zg;          // [T,B,4H] in: gates ; out: d loss / d a
  const float* R;     // [H,4H]
  const float* c;     // [T,B,H]
  const float* c0;    // [B,H] or null
  const float* dy;    // [T,B,ldy], offset to this direction's columns
  const float* dhT;   // [B,H] or null
  const float* dcT;   // [B,H] or null
  float* dh0;         // [B,H] or null
  float* dc0;         // [B,H] or null
  float* db;          // [4H]
  int direction;
};
struct RecShape {
  int T, B, H, ldy, ndir, operand_dtype;
  // tuning of the persistent engine (0 = chosen per shape)
  int batch_groups = 0;   // groups the sequences are dealt out to per direction
  int bwd_exchange = 0;   // exchanges per step of the backward pass: 1 two (d a_t out, partial tiles back), 2 one where it applies
  bool fp32_instructions = false;   // fp32 operands: keep to the fp32 matrix instructions (no three-part kernels)
};

// Scratch bytes the recurrent passes need (max over both engines, fwd and bwd).
size_t rec_workspace_bytes(const RecShape& s);
// the part of it that the forward pass uses (a prefix of the same layout)
size_t rec_workspace_bytes_fwd(const RecShape& s);
// true if the persistent kernels can hold this shape (LDS, grid <= CUs).
bool rec_persistent_supported(const RecShape& s, int num_cus, size_t max_lds);

// [s_begin, s_end): the steps of the pass (in processing order) that this call enqueues; a pass may
// be split into consecutive calls on one stream that together cover [0, T) (persistent engine only;
// the stepwise engine takes the whole range).  The scratch carries the state from call to call.
hipError_t rec_forward(hipStream_t stream, const RecShape& s, const RecFwdDir* dirs,
                       const int32_t* seq_lens, void* ws, unsigned* flag, bool persistent, int* resident_err,
                       int s_begin, int s_end);
hipError_t rec_backward(hipStream_t stream, const RecShape& s, const RecBwdDir* dirs,
                        const int32_t* seq_lens, void* ws, unsigned* flag, bool persistent, int* resident_err,
                        int s_begin, int s_end);

// the two engines behind rec_forward / rec_backward
bool persistent_supported(const RecShape& s, int num_cus, size_t max_lds);
size_t persistent_scratch_bytes(const RecShape& s);
// LDS a workgroup of the persistent kernels requests (larger of forward / backward); 0: shape not supported
size_t persistent_lds_bytes(const RecShape& s, int num_cus, size_t max_lds);
// LDS of the matrix-product kernel that can share a CU with other work (128 x 128 tiles)
size_t gemm_small_lds_bytes(int operand_dtype, int variant);
// {groups, sequences per group, rows a group can hold, units per workgroup, forward members, backward members, Hp,
//  Hq (two exchanges) or padded H of the backward product (one), exchanges per backward step, 0}
bool persistent_plan_info(const RecShape& s, int num_cus, size_t max_lds, int out[10]);
// scratch of the forward pass alone (the backward pass may need more)
size_t persistent_scratch_bytes_fwd(const RecShape& s);
// test hook: workgroup `mute_workgroup` (-1: none) withholds its step flags; wait bound in 100 MHz ticks (0: default)
void persistent_test_hook(int mute_workgroup, unsigned long long wait_ticks);
// workgroup `slow_workgroup` of every persistent launch publishes each step `ticks` of the 100 MHz clock late (-1: none)
void persistent_test_delay(int slow_workgroup, unsigned ticks);
hipError_t persistent_forward(hipStream_t stream, const RecShape& s, const RecFwdDir* dirs, const int32_t* seq_lens,
                              char* scratch, unsigned* err, int* resident_err, int s_begin, int s_end);
hipError_t persistent_backward(hipStream_t stream, const RecShape& s, const RecBwdDir* dirs, const int32_t* seq_lens,
                               char* scratch, unsigned* err, int* resident_err, int s_begin, int s_end);
size_t stepwise_scratch_floats_per_dir(const RecShape& s);
hipError_t stepwise_forward(hipStream_t stream, const RecShape& s, const RecFwdDir* dirs, const int32_t* seq_lens,
                            float* const* buf);
hipError_t stepwise_backward(hipStream_t stream, const RecShape& s, const RecBwdDir* dirs, const int32_t* seq_lens,
                             float* const* buf);

// dR += h0^T * dz(first processed valid frame of each sequence)
hipError_t add_h0_outer(hipStream_t stream, int T, int B, int H, int direction, const float* h0,
                        const float* dz, const int32_t* seq_lens, float* dR);
// column sums of a [rows, cols] matrix (stepwise engine's bias gradient)
hipError_t column_sum(hipStream_t stream, const float* a, size_t rows, int cols, int lda, float* out);
// plain copy kernel (counter calibration)
hipError_t copy_f32(hipStream_t stream, float* dst, const float* src, size_t n);
// zero the timeout flag
hipError_t clear_flag(hipStream_t stream, unsigned* flag);

// ---------------------------------------------------------------------------
// Two-dimensional LSTM layer: the scans over the anti-diagonals (mdlstm.hip).
// P = Hh * Ww * B pixel slots, pixel (u, v) of image n at index (u * Ww + v) * B + n.
// ---------------------------------------------------------------------------
struct MdShape { int Hh, Ww, B, H, S; };   // S: row stride of the hc arrays (>= 2H, multiple of 4)
struct MdDir {
  float* zg;          // [P, 5H] in: b + x W ; forward out: gates i|f_u|f_v|o|g ; backward out: d loss / d a
  float* c;           // [P, H]
  float* hc;          // [P, S] forward out: h of the vertical | horizontal predecessor of every pixel (| x, see mdlstm_copy_x)
  const float* Ru;    // [H, 5H]
  const float* Rv;    // [H, 5H]
};
bool mdlstm_supported(const MdShape& s);
// test hook: workgroup `mute_workgroup` (-1: none) hands no row on; wait bound in 100 MHz ticks (0: default)
void mdlstm_test_hook(int mute_workgroup, unsigned long long wait_ticks);
// dirs[4] in the order (du, dv) = (+,+), (+,-), (-,+), (-,-); y, dy: [P, 4H]
// halo: mdlstm_halo_words() 64-bit words of scratch (rows handed between bands); err: timeout flag
size_t mdlstm_halo_words(const MdShape& s);
// x1 != null: the input has one value per pixel; zg is not read, the input part is formed in the kernel from x1 [P],
// W1[4] ([1, 5H] each) and b1[4] ([5H]), and x1 is written into column 2H of the hc arrays (S >= 2H + 1)
hipError_t mdlstm_forward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths, float* y,
                          unsigned long long* halo, unsigned* err, const float* x1 = nullptr,
                          const float* const* W1 = nullptr, const float* const* b1 = nullptr);
// x into columns [2H, 2H + D) of the four hc arrays (S >= 2H + D)
hipError_t mdlstm_copy_x(hipStream_t stream, const MdShape& s, const MdDir* dirs, const float* x, int D);
// rows [0,H), [H,2H), [2H,2H+D) of four stacked [2H + D, 5H] gradients to dRu, dRv, dW
hipError_t mdlstm_scatter_grads(hipStream_t stream, int D, int H, const float* const* stacked, float* const* dRu,
                                float* const* dRv, float* const* dW);
// dbpart: scratch of mdlstm_dbpart_floats(); db[4]: bias gradients [5H] per direction
size_t mdlstm_dbpart_floats(const MdShape& s);
hipError_t mdlstm_backward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths, const float* dy,
                           float* dbpart, float* const* db, unsigned long long* halo, unsigned* err);

// the stepwise engine of the two-dimensional layer (mdlstm_stepwise.hip): one launch per anti-diagonal, any shape;
// zg must hold b + x W (there is no in-kernel input path); scratch: mdlstm_stepwise_scratch_floats() floats
size_t mdlstm_stepwise_scratch_floats(const MdShape& s);
hipError_t mdlstm_stepwise_forward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths, float* y);
hipError_t mdlstm_stepwise_backward(hipStream_t stream, const MdShape& s, const MdDir* dirs, const int32_t* widths,
                                    const float* dy, float* scratch, float* const* db);

// output layer and updates (output_layer.hip).  z: [T*B, ld], logits in columns [0, C) in, d loss / d logits out with
// columns [C, ld) zeroed; scratch: ce_scratch_floats(); loss, errors: one value each; dbo: [C] column sums of the result
size_t ce_scratch_floats(int rows, int C);
hipError_t softmax_ce_rows(hipStream_t stream, float* z, int ld, const int32_t* labels, const int32_t* seq_lens, int T, int B,
                           int C, float* scratch, float* loss, int32_t* errors, float* dbo);
// dst[r, 0..cols_dst) = src[r, 0..cols_src) followed by zeros
hipError_t repitch(hipStream_t stream, const float* src, int ld_src, int cols_src, float* dst, int ld_dst, int cols_dst, int rows);
hipError_t sgd_momentum(hipStream_t stream, float* p, const float* g, float* v, size_t n, float lr, float mu);
hipError_t adam(hipStream_t stream, float* p, const float* g, float* m, float* v, size_t n, double lr, double b1, double b2,
                double eps, int step);

// streaming mode (stream.hip): out[s * B + b] = clamp(seq_lens[b] - s * Tc, 0, Tc); dst (+)= src; fill
hipError_t segment_lens(hipStream_t stream, const int32_t* seq_lens, int B, int S, int Tc, int32_t* out);
hipError_t accumulate(hipStream_t stream, float* dst, const float* src, size_t n, bool assign);
hipError_t fill_f32(hipStream_t stream, float* dst, size_t n, float v);

// chunking (chunking.hip): segment table on the host, gather of the segments into a minibatch on the device
long long chunk_plan(const int32_t* seq_lens, int B, int size, int step, int32_t* seq, int32_t* start, int32_t* len,
                     long long max_chunks);
hipError_t chunk_gather(hipStream_t stream, const float* x, int T, int B, int D, int ldx, const int32_t* seq,
                        const int32_t* start, const int32_t* len, int nchunks, int size, float* xc);

// bare exchange of the persistent kernels' step chain (measurement aid, see exchange_probe.hip)
size_t exchange_probe_bytes(int groups, int members, int tile_bytes);
hipError_t exchange_probe(hipStream_t stream, int groups, int members, int tile_bytes, int read_bytes, int steps,
                          void* ws, float* us_per_step, int* timed_out, int* resident_err);

struct DeviceInfo { int num_cus; size_t max_lds; };
hipError_t device_info(DeviceInfo* out);

}  // namespace rlstm
