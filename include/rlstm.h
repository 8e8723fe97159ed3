/*
 * rlstm.h - C ABI of the MI355X (gfx950) LSTM / deep BLSTM training kernels.
 *
 * The library implements the LSTM layer of RETURNN (arXiv 1608.00895) as the
 * paper's Sec. 4.2 describes it: the non-recurrent part of the forward pass is
 * one matrix product over all frames of the minibatch, the recurrent part runs
 * through time with a fused gating step, back-propagation first runs back
 * through time and then forms the weight and input gradients as whole-minibatch
 * matrix products, and buffers are reused in place.  Tensors are time-major
 * [time, batch, feature] with a per-(time, batch) validity mask (Sec. 5),
 * given here as seq_lens[B]: frame t of sequence n is valid iff t < seq_lens[n].
 * A layer has a direction (+1 scans t = 0..T-1, -1 scans t = T-1..0) and a
 * bidirectional layer feeds [y_forward | y_backward] to the next layer (Fig. 1).
 * Gradients are plain sums over frames and sequences (Sec. 4.3).
 *
 * Cell (the paper cites the LSTM without printing equations; this is the
 * reading fixed for the whole library).  With a = b + x_t W + h_prev R, a 4H
 * wide row whose column blocks are  i | f | o | g  in that order:
 *     i = s(a_i)  f = s(a_f)  o = s(a_o)  g = tanh(a_g)     s(u) = 1/(1+exp(-u))
 *     c~ = f*c_prev + i*g        h~ = o*tanh(c~)
 *     valid frame:   (h, c) <- (h~, c~),  y_t = h~
 *     invalid frame: (h, c) unchanged,    y_t = 0
 * "prev" is the previously processed frame in the layer's direction; the state
 * before the first processed frame is (h0, c0).  c[t] returns the carried cell
 * state after frame t.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers (HIP, fp32 unless said otherwise,
 *     16-byte aligned recommended) owned by the caller.  Descriptors are HOST
 *     structs.  The library allocates and frees no device memory and only
 *     enqueues work on the streams passed in (a null stream handle is HIP's
 *     default stream).  It never synchronises the device, with two exceptions
 *     that say so: rlstm_last_timeout() and the measurement aid
 *     rlstm_exchange_floor().
 *   - Inputs are read-only.  Outputs are overwritten, never accumulated into.
 *   - workspace must hold rlstm_workspace_bytes() (resp. rblstm_workspace_bytes())
 *     bytes; its contents need no initialisation and are undefined afterwards.
 *     Calls that share a workspace must not overlap in time.
 *   - Return value: 0 on success, a negative RLSTM_E* code otherwise; nothing
 *     is enqueued when an argument check fails.  rlstm_strerror() names a code.
 *   - seq_lens values are clamped on the device to [0, T].
 *   - The recurrent kernels are persistent: all of their workgroups must be
 *     resident at once, so the call fails with RLSTM_ERESIDENT when the device
 *     cannot hold them.  Their waits on each other are bounded; if one ever
 *     expires the kernel stops stepping and raises a flag in the first word of
 *     the workspace that rlstm_last_timeout() reports.  The flag is cleared by
 *     the entry points that start a pass (lstm_fwd, blstm_stack_fwd,
 *     blstm_stack_fwd_bwd, lstm_stream_fwd_bwd, mdlstm_fwd) and by nothing else:
 *     the backward entry points (lstm_bwd, blstm_stack_bwd, mdlstm_bwd) leave it,
 *     and their recurrent kernels do nothing while it is raised, so one read
 *     after the backward call tells about both passes.  The backward entry
 *     points must therefore be given the workspace of the forward call.
 */
#ifndef RLSTM_H
#define RLSTM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define RLSTM_API __attribute__((visibility("default")))
#else
#define RLSTM_API
#endif

#define RLSTM_OK          0
#define RLSTM_ENULL      -1   /* a required pointer is null */
#define RLSTM_EDIM       -2   /* a dimension is <= 0 or a leading dimension is too small */
#define RLSTM_EMODE      -3   /* bad direction / operand_dtype / engine */
#define RLSTM_ESIZE      -4   /* a workspace passed with its size is too small */
#define RLSTM_ERESIDENT  -5   /* persistent kernel cannot be made co-resident / shape unsupported by the engine */
#define RLSTM_EHIP       -6   /* a HIP runtime call failed */

#define RLSTM_ENGINE_AUTO        0  /* persistent kernels where the shape fits on chip, else stepwise */
#define RLSTM_ENGINE_PERSISTENT  1  /* one launch runs all T steps; fails if the shape does not fit */
#define RLSTM_ENGINE_STEPWISE    2  /* one launch per time step (plain kernels; any shape) */

/* One LSTM layer, one direction.  Host struct, all int32. */
typedef struct rlstm_desc {
  int32_t T;              /* padded length (frames)                                   */
  int32_t B;              /* sequences in the minibatch                               */
  int32_t D;              /* input feature width                                      */
  int32_t H;              /* units                                                    */
  int32_t direction;      /* +1 or -1 (Fig. 1)                                        */
  int32_t operand_dtype;  /* 0: fp32; 1: matrix-product operands rounded to bf16,
                             fp32 accumulation, fp32 cell state and outputs          */
  int32_t ldx;            /* row stride (floats) of x and dx, >= D; 0 means D         */
  int32_t ldy;            /* row stride (floats) of y and dy, >= H; 0 means H         */
  int32_t engine;         /* RLSTM_ENGINE_*                                           */
  /* Tuning (see "Tuning fields" below); 0 = library default for every field.              */
  int32_t batch_groups;   /* groups the sequences are dealt out to per direction      */
  int32_t bwd_exchange;   /* exchanges per step of the backward recurrent kernel      */
  int32_t gemm_variant;   /* which fp32 matrix-product kernel                         */
} rlstm_desc;

/*
 * Tuning fields of the descriptors.  They select among implementations of the same computation: results never
 * differ beyond the order of floating-point sums.  0 always means "library default"; a value outside the ranges
 * below is RLSTM_EMODE.  They travel with the descriptor, so that callers with different shapes (or threads) in one
 * process tune independently; the library keeps no tuning state.
 *   batch_groups  0, 1, 2, 4 or 8.  The sequences of a minibatch are independent; the persistent engine deals them
 *                 out to this many groups of workgroups per direction, each with its own copy of the recurrent
 *                 matrix, which exchange h_t / d a_t only among themselves (directions * groups <= 8; a value the
 *                 shape cannot use makes the persistent engine unavailable for it).  Default: chosen per shape.
 *   bwd_exchange  1: two exchanges between workgroups per step of the pass back through time (Sec. 4.2) - workgroups
 *                 fetch a quarter of d a_t each, multiply it with their rows of R^T and hand partial tiles to the
 *                 owners of the units;  2: one exchange per step where it applies (groups of at most 16 sequences,
 *                 fp32, H <= 512) - every workgroup multiplies its own columns of d a_t with its rows of R^T and
 *                 hands a piece of the result to every other workgroup of its group, which adds the pieces in a
 *                 fixed order.  Default: 1.
 *   gemm_variant  which kernel multiplies fp32 operands (Sec. 4.2's products over the whole minibatch).  Default (0):
 *                 each operand value is cut, exactly, into three bf16 parts (8 + 8 + 8 of its 24 significant bits) on
 *                 its way into LDS, and the six largest of the nine part products are summed in fp32 by the bf16 matrix
 *                 instructions; what is left out is below 2^-21 of each term, and against an fp64 product the result is
 *                 as close as that of the fp32 matrix instructions (an infinity among the operands gives NaN).
 *                 1, 2, 3: the fp32 matrix instructions - 1 the pipelined kernel wherever its operand conditions hold
 *                 (both operands made of whole, 16-byte aligned float4s), 2 the plain kernel, 3 the pipelined kernel
 *                 where its conditions hold and the product does not run beside the recurrent kernels on the same CUs.
 *                 Products of bf16 operands (operand_dtype 1) ignore 3.
 *                 The recurrent kernels follow: with fp32 operands and groups of more than 16 sequences (two or
 *                 more 16-row tiles per workgroup, H <= 512) they exchange h_t / d a_t and keep R as three bf16
 *                 parts each and form the recurrent product the same way; 1, 2 and 3 keep them on the fp32 matrix
 *                 instructions.  Groups of up to 16 sequences always use those.
 *   first_piece   (stack descriptors) with two streams and the persistent engine each layer's recurrent pass is cut
 *                 into pieces of first_piece, first_piece, 2 first_piece, 4 first_piece, ... steps, and the matrix
 *                 product that feeds a piece runs on stream b while stream a is inside the piece before it.
 *                 -1: passes are not cut.  Default: 128.
 *   overlap_mode  (stack descriptors) 1: matrix products and recurrent passes one after the other;  2: products
 *                 and recurrent workgroups share CUs and the passes are cut into pieces (falls back to 1 where the
 *                 two LDS footprints do not fit one CU).  Default: chosen per shape.
 */

/* Deep bidirectional stack: L layers, each a forward and a backward LSTM of H
 * units on the same input; layer 0 reads D features, layers >= 1 read 2H. */
typedef struct rblstm_desc {
  int32_t L, T, B, D, H;
  int32_t operand_dtype;  /* as in rlstm_desc */
  int32_t engine;         /* RLSTM_ENGINE_* */
  int32_t first_piece, batch_groups, overlap_mode, gemm_variant, bwd_exchange;   /* tuning, 0 = default */
} rblstm_desc;

/* Bytes of the opaque forward-to-backward buffer of lstm_fwd / lstm_bwd (it
 * holds the activated gates [T,B,4H]); 0 if the descriptor is invalid. */
RLSTM_API size_t rlstm_reserve_bytes(const rlstm_desc* desc);
/* Bytes of scratch for lstm_fwd / lstm_bwd; 0 if the descriptor is invalid. */
RLSTM_API size_t rlstm_workspace_bytes(const rlstm_desc* desc);
/* Same for blstm_stack_fwd_bwd (reserve: per layer and direction the gate
 * buffer [T,B,4H] and cell buffer [T,B,H], plus the outputs [T,B,2H] of all layers
 * but the top one, whose output is the caller's y_top). */
RLSTM_API size_t rblstm_reserve_bytes(const rblstm_desc* desc);
RLSTM_API size_t rblstm_workspace_bytes(const rblstm_desc* desc);

/*
 * lstm_fwd - forward pass of one layer in one direction (Sec. 4.2: one matrix
 * product x W for all T*B frames, then the recurrence with fused gating;
 * Sec. 5 mask; Fig. 1 direction).
 *   x   [T,B,ldx]  in     W [D,4H] in    R [H,4H] in    b [4H] in
 *   h0, c0 [B,H]   in, may be null (= zeros)
 *   seq_lens [B]   in, int32
 *   y   [T,B,ldy]  out (only the first H floats of each row are written)
 *   c   [T,B,H]    out, carried cell state after each frame
 *   hT, cT [B,H]   out, may be null: state after the last processed frame
 *   reserve        out, rlstm_reserve_bytes(): needed by lstm_bwd
 */
RLSTM_API int lstm_fwd(const rlstm_desc* desc, const float* x, const float* W, const float* R, const float* b,
             const float* h0, const float* c0, const int32_t* seq_lens,
             float* y, float* c, float* hT, float* cT,
             void* reserve, void* workspace, void* hip_stream);

/*
 * lstm_bwd - back-propagation through time for the pass lstm_fwd recorded
 * (Sec. 4.2: the recurrent part is propagated back through time first, then
 * the gradients w.r.t. weights and inputs are whole-minibatch matrix
 * products; Sec. 4.3: unscaled sums).
 *   x, W, R, seq_lens, h0, c0  as given to lstm_fwd
 *   y, c                       as written by lstm_fwd
 *   reserve                    in/out: consumed (holds d loss / d a afterwards)
 *   workspace                  the one given to lstm_fwd (its first word carries the timeout flag)
 *   dy  [T,B,ldy]  in, gradient w.r.t. y (rows beyond a sequence's length are ignored)
 *   dhT, dcT [B,H] in, may be null (= zeros): gradient w.r.t. hT, cT
 *   dx  [T,B,ldx]  out, may be null (skipped); 0 at invalid frames
 *   dW [D,4H], dR [H,4H], db [4H]  out
 *   dh0, dc0 [B,H] out, may be null
 */
RLSTM_API int lstm_bwd(const rlstm_desc* desc, const float* x, const float* W, const float* R,
             const int32_t* seq_lens, const float* h0, const float* c0,
             const float* y, const float* c, void* reserve,
             const float* dy, const float* dhT, const float* dcT,
             float* dx, float* dW, float* dR, float* db, float* dh0, float* dc0,
             void* workspace, void* hip_stream);

/*
 * lstm_fwd_noalloc - lstm_fwd for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and results as lstm_fwd (the same kernels run) without `workspace`: the scratch of the
 * recurrent pass (timeout flag, step flags, exchange arrays, carried state) lives in a device array
 * of RLSTM_NOALLOC_SCRATCH_LIMIT bytes inside the library, one copy per GPU, held until the process
 * ends.  The call allocates nothing (no hipMalloc / hipFree, no events: the timing hooks of
 * rlstm_profile_enable() are skipped) and clears what must start at zero with kernels, not memsets.
 *   rlstm_noalloc_scratch_bytes(desc): scratch this shape needs (0: invalid descriptor);
 *   shapes that need more than RLSTM_NOALLOC_SCRATCH_LIMIT are refused with RLSTM_ESIZE
 *   (H = 512, B = 64 needs about 10 MiB).
 * All calls on one GPU share that GPU's array, which keeps the last call's contents: calls that
 * overlap in time on one GPU (different streams or threads) race and must be serialised by the
 * caller.  The timeout flag is read with rlstm_last_timeout_on(NULL, stream).
 */
#define RLSTM_NOALLOC_SCRATCH_LIMIT ((size_t)16 << 20)
RLSTM_API size_t rlstm_noalloc_scratch_bytes(const rlstm_desc* desc);
RLSTM_API int lstm_fwd_noalloc(const rlstm_desc* desc, const float* x, const float* W, const float* R, const float* b,
             const float* h0, const float* c0, const int32_t* seq_lens,
             float* y, float* c, float* hT, float* cT, void* reserve, void* hip_stream);

/*
 * blstm_stack_fwd_bwd - one training pass (forward, then backward) of an
 * L-layer bidirectional LSTM stack with zero initial states (Fig. 1 stacking,
 * Sec. 4.2 kernels).  The two directions of a layer run concurrently.
 *   x [T,B,D] in;  seq_lens [B] in
 *   params: HOST array of 6*L DEVICE pointers, for layer l and direction d
 *           (0 forward, 1 backward): params[6l+3d+0] = W [D_l,4H],
 *           +1 = R [H,4H], +2 = b [4H];  D_0 = D, D_l = 2H otherwise
 *   dy_top [T,B,2H] in: gradient of the loss w.r.t. the top layer's output
 *   y_top  [T,B,2H] out
 *   grads:  HOST array of 6*L DEVICE pointers laid out like params (dW, dR, db), out
 *   dx [T,B,D] out, may be null (the bottom layer's input gradient is skipped)
 *   stream_a carries the dependent chain; stream_b, if not null and different,
 *   is used to overlap independent weight-gradient products with the next
 *   layer's pass back through time.  On return all work has been enqueued and
 *   stream_a waits for everything placed on stream_b.
 */
RLSTM_API int blstm_stack_fwd_bwd(const rblstm_desc* desc, const float* x, const float* const* params,
                        const int32_t* seq_lens, const float* dy_top,
                        float* y_top, float* const* grads, float* dx,
                        void* reserve, void* workspace, void* hip_stream_a, void* hip_stream_b);

/*
 * blstm_stack_bwd - the backward half alone: the same arguments, after a blstm_stack_fwd (or
 * blstm_stack_fwd_bwd) call with the same descriptor, x, params, seq_lens, reserve and workspace
 * whose y_top is passed back in.  This is the form a loss layer on top of the stack needs, whose
 * dy_top depends on y_top (softmax_ce_fwd_bwd below).  dy_top must be complete in stream_a's order.
 */
RLSTM_API int blstm_stack_bwd(const rblstm_desc* desc, const float* x, const float* const* params,
                    const int32_t* seq_lens, const float* dy_top, const float* y_top,
                    float* const* grads, float* dx,
                    void* reserve, void* workspace, void* hip_stream_a, void* hip_stream_b);

/* Forward half only of the stack (inference / parity of hidden layers):
 * same arguments as above without gradients. */
RLSTM_API int blstm_stack_fwd(const rblstm_desc* desc, const float* x, const float* const* params,
                    const int32_t* seq_lens, float* y_top,
                    void* reserve, void* workspace, void* hip_stream_a);

/*
 * rlstm_gemm_f32 - the whole-minibatch matrix product the layer is built on
 * (Sec. 4.2: the non-recurrent part of all frames of a minibatch is one product), exposed
 * for measurement and testing:  C[M,N] = op(A) op(B) (+ bias[n] on every row).
 *   trans_a == 0: A is [M,K] with row stride lda;  != 0: A is stored [K,M]
 *   trans_b == 0: B is [K,N] with row stride ldb;  != 0: B is stored [N,K]
 *   C [M,N] out, row stride ldc; bias [N] or null
 *   variant: the gemm_variant tuning value (0 = default)
 *   splitk_ws: scratch of splitk_ws_bytes (may be null / 0): lets products with
 *   K much larger than M, N split K into slices that are summed in a fixed order.
 */
RLSTM_API int rlstm_gemm_f32(int trans_a, int trans_b, int M, int N, int K,
                   const float* A, int lda, const float* B, int ldb, float* C, int ldc,
                   const float* bias, int variant, void* splitk_ws, size_t splitk_ws_bytes, void* hip_stream);
/* Same product with both operands rounded to bf16 (round to nearest even) and fp32
 * accumulation; A, B, C and bias stay fp32 in memory (the operand_dtype = 1 variant). */
RLSTM_API int rlstm_gemm_bf16(int trans_a, int trans_b, int M, int N, int K,
                    const float* A, int lda, const float* B, int ldb, float* C, int ldc,
                    const float* bias, int variant, void* splitk_ws, size_t splitk_ws_bytes, void* hip_stream);

/*
 * The bf16-operand products of the stack entry points read their operands from bf16 COPIES (half the bytes, no
 * rounding inside the product), each stored so that the product walks along its rows: x, every layer's output and
 * d a both as stored and transposed, W as stored and transposed.  The copies live in the stack's workspace when
 * operand_dtype is 1.  The three calls below expose that path for measurement and testing.
 *   rlstm_to_bf16: dst[i] = bf16(src[i]), round to nearest even; n a multiple of 8, both arrays 16-byte aligned
 *   (RLSTM_EDIM otherwise).
 *   rlstm_to_bf16_2d: src [R, C] fp32 with row stride ld -> dst [R, C] bf16 (may be null) and dst_t [C, R] bf16, its
 *   transpose (may be null), both dense; R, C multiples of 8, ld a multiple of 4, all arrays 16-byte aligned
 *   (RLSTM_EDIM otherwise).
 *   rlstm_gemm_bf16_mem: C[M,N] = op(A16) op(B16) (+ bias), fp32 accumulation, operands bf16 in memory with the
 *   trans_a / trans_b / lda / ldb meaning of rlstm_gemm_f32 (strides in bf16 elements).  The result has the bits of
 *   rlstm_gemm_bf16 on fp32 operands that round to these bf16 values.  RLSTM_EMODE when the shape does not take the
 *   kernel that reads bf16 from memory (it needs 256 x 256 tiles to fill the chip, whole 16-byte aligned groups of 8
 *   values along the operands' contiguous dimensions and K a multiple of 8).  variant 0: one workgroup per CU that
 *   walks through its share of the tiles; operands that are both laid out along k (trans_a == 0, trans_b != 0) go
 *   through a ring of LDS slabs filled by buffer loads that write LDS directly.  For measurement: 3, one workgroup
 *   per tile; 4, slabs staged through registers for every layout.  Other values: RLSTM_EMODE.
 */
RLSTM_API int rlstm_to_bf16(uint16_t* dst, const float* src, size_t n, void* hip_stream);
RLSTM_API int rlstm_to_bf16_2d(uint16_t* dst, uint16_t* dst_t, const float* src, int R, int C, int ld, void* hip_stream);
RLSTM_API int rlstm_gemm_bf16_mem(int trans_a, int trans_b, int M, int N, int K,
                        const uint16_t* A16, int lda, const uint16_t* B16, int ldb,
                        float* C, int ldc, const float* bias, int variant, void* splitk_ws, size_t splitk_ws_bytes, void* hip_stream);

/*
 * Optional per-kernel timing for measurement (not part of the method).  While
 * enabled, every kernel group the library enqueues is bracketed by a pair of
 * HIP events on the stream it is launched on.  rlstm_profile_read() waits for
 * the recorded events, writes up to max_entries entries (in launch order) and
 * clears the record; it returns the number of entries recorded (which may
 * exceed max_entries) or a negative code; when timing has been switched off it
 * also destroys the events it had created.  Not thread-safe.
 *   kind: 0 input projection X W + b        1 recurrent forward pass
 *         2 pass back through time          3 input gradient dZ W^T
 *         4 weight gradient X^T dZ          5 recurrent weight gradient Hprev^T dZ
 *         6 product of the output layer     7 softmax / cross-entropy rows and their sums
 *   layer: stack layer (0 for the single-layer entry points); ndir: directions covered;
 *   steps: recurrent steps the group covers (a pass may be cut into several groups; 0 for a
 *   matrix product); flop: algorithmic floating-point operations of the group (2 M N K of a
 *   product; 2 B H 4H per step and direction of a recurrent pass)
 */
typedef struct rlstm_profile_entry {
  int32_t kind, layer, ndir, steps;
  float ms, reserved;
  double flop;
} rlstm_profile_entry;
RLSTM_API int rlstm_profile_enable(int on);
RLSTM_API int rlstm_profile_read(rlstm_profile_entry* out, int max_entries);

/*
 * rlstm_copy_f32 - plain device-to-device copy kernel of n floats (one float4 per
 * thread, grid-stride).  Measurement utility: a kernel of exactly known HBM traffic
 * (4n bytes read, 4n bytes written) against which hardware counters are scaled.
 */
RLSTM_API int rlstm_copy_f32(float* dst, const float* src, size_t n, void* hip_stream);

/* Reads (with a blocking device-to-host copy) the timeout flag that the
 * persistent kernels keep at the start of `workspace`: 0 = no bounded wait
 * expired since the last forward entry point that used this workspace, 1 = one
 * did and the results are invalid, negative = RLSTM_E* code.  The flag is not
 * changed.  rlstm_last_timeout synchronises the DEVICE first;
 * rlstm_last_timeout_on waits only for `hip_stream` (the stream the calls in
 * question were enqueued on: for the stack entry points stream a) and, given a
 * null workspace, reads the flag of lstm_fwd_noalloc on the current device. */
RLSTM_API int rlstm_last_timeout(const void* workspace);
RLSTM_API int rlstm_last_timeout_on(const void* workspace, void* hip_stream);


/*
 * Two-dimensional (multidimensional) LSTM layer with four scan directions (Sec. 4.2: the state of
 * pixel (u, v) depends on the states of its two predecessors (u-1, v) and (u, v-1) in scan order;
 * all pixels of an anti-diagonal are computed together; the four directions and all images of the
 * batch run at once).  The paper names the cell by citation only; the cell used is the
 * multidimensional LSTM with one forget gate per dimension:
 *     a  = b + x(u,v) W + h(u',v) R_u + h(u,v') R_v          5H wide, blocks i | f_u | f_v | o | g
 *     c~ = f_u * c(u',v) + f_v * c(u,v') + i * g ,   h~ = o * tanh(c~)
 * with (u', v') the predecessor row / column of the scan direction, sigmoid on i, f_u, f_v, o, tanh
 * on g.  A predecessor outside the image contributes zero state.  All images have Hh rows; image n
 * has widths[n] columns (clamped to [0, Ww]); a pixel at or beyond its image's width is outside the
 * image (y = 0 there, no influence on anything), so every image is processed as if alone.
 * Directions, in this order: (du, dv) = (+1,+1), (+1,-1), (-1,+1), (-1,-1).
 *
 * Layouts (device memory, fp32, row-major): x [Hh, Ww, B, D]; y, dy [Hh, Ww, B, 4H] (the four
 * directions' outputs side by side in the order above); params / grads: 16 pointers, per direction
 * W [D, 5H], R_u [H, 5H], R_v [H, 5H], b [5H]; widths [B] int32.  Gradients are plain sums and
 * are overwritten.  dx [Hh, Ww, B, D] may be null.  reserve (rmdlstm_reserve_bytes) carries the
 * gates, cell states and predecessor outputs from mdlstm_fwd to mdlstm_bwd, which overwrites it;
 * workspace (rmdlstm_workspace_bytes) is scratch.  The caller owns all buffers; nothing is
 * allocated and the device is not synchronised.
 * Engines (the `engine` field, RLSTM_ENGINE_* as for the one-dimensional layer).  PERSISTENT: one launch per pass;
 * the rows of a scan are dealt out to workgroups in bands of 16 that hand one row per anti-diagonal to their
 * neighbour through the workspace; all such waits are bounded (2 s) and rlstm_last_timeout(workspace) tells
 * whether one expired (the results are then invalid); limits Hh <= 256, H <= 32 (RLSTM_ERESIDENT beyond them, and
 * the size queries return 0).  STEPWISE: one launch per anti-diagonal with plain kernels, any shape.  AUTO:
 * PERSISTENT where the shape fits, else STEPWISE.  operand_dtype must be 0.  Other errors as for lstm_fwd.
 */
typedef struct rmdlstm_desc {
  int32_t Hh, Ww, B, D, H;
  int32_t operand_dtype;      /* 0 (fp32) */
  int32_t engine;             /* RLSTM_ENGINE_* */
} rmdlstm_desc;
RLSTM_API size_t rmdlstm_reserve_bytes(const rmdlstm_desc* d);
RLSTM_API size_t rmdlstm_workspace_bytes(const rmdlstm_desc* d);
RLSTM_API int mdlstm_fwd(const rmdlstm_desc* d, const float* x, const float* const* params, const int32_t* widths,
                         float* y, void* reserve, void* workspace, void* hip_stream);
RLSTM_API int mdlstm_bwd(const rmdlstm_desc* d, const float* x, const float* const* params, const int32_t* widths,
                         void* reserve, const float* dy, float* dx, float* const* grads, void* workspace,
                         void* hip_stream);

/*
 * Chunking (Sec. 4: sequences whose lengths differ a lot are cut into segments of constant
 * length, possibly overlapping, so that a minibatch carries little zero padding, at the price of
 * the context across segment borders; Sec. 6 trains on segments of 250 frames, zero-padded where a
 * sequence ends, 81 per batch).
 *
 * rlstm_chunk_plan (host, integers only): the segments of a sequence of n = seq_lens[b] frames
 * start at frames 0, step, 2*step, ... (every start < n) and hold min(size, n - start) frames.
 * Writes, sequence by sequence with starts ascending, for chunk k: chunk_seq[k] = b,
 * chunk_start[k], chunk_len[k] (host arrays of max_chunks entries; any may be null) and returns
 * the number of segments, which may exceed max_chunks (then only the first max_chunks entries were
 * written), or a negative code.
 *
 * rlstm_chunk_gather (device): xc[t, k, :] = x[chunk_start[k] + t, chunk_seq[k], :] for
 * t < chunk_len[k], else 0; x [T, B, ldx] (ldx = 0 means D), xc [size, n_chunks, D], the three
 * tables are device arrays of n_chunks entries.  chunk_len is the seq_lens of the minibatch xc.
 * Table entries that point outside x are treated as padding.
 */
RLSTM_API long long rlstm_chunk_plan(const int32_t* seq_lens, int B, int size, int step, int32_t* chunk_seq,
                                     int32_t* chunk_start, int32_t* chunk_len, long long max_chunks);
RLSTM_API int rlstm_chunk_gather(const float* x, int T, int B, int D, int ldx, const int32_t* chunk_seq,
                                 const int32_t* chunk_start, const int32_t* chunk_len, int n_chunks, int size,
                                 float* xc, void* hip_stream);

/*
 * Streaming mode: a unidirectional (direction +1) stack of L LSTM layers reads its sequences in S
 * consecutive segments of Tc frames; every layer starts a segment from the final state it reached
 * in the segment before (Sec. 3.2: final states handed on from one recurrent layer to another),
 * so the forward result is that of the uncut sequences and the context that plain cutting into
 * segments gives up (Sec. 4) is kept.  Back-propagation through time is truncated at the segment
 * boundaries: the backward pass of a segment takes the segment's initial state as a constant,
 * no gradient arrives at its final state, and the gradients of the segments are summed.  Memory:
 * one segment of activations, whatever S is.  Calling with S = 1 once per segment, passing the
 * same `state` array every time, streams a sequence of any length (and lets a loss layer run
 * between the calls).
 *   x [S*Tc,B,D] in; seq_lens [B] in: lengths of the whole sequences (segment s holds
 *   clamp(len - s*Tc, 0, Tc) valid frames of a sequence; a sequence that has ended keeps its state)
 *   params: HOST array of 3*L DEVICE pointers: params[3l] = W [D_l,4H], +1 = R [H,4H], +2 = b [4H];
 *           D_0 = D, D_l = H otherwise
 *   dy_top [S*Tc,B,H] in; y_top [S*Tc,B,H] out
 *   grads: HOST array of 3*L DEVICE pointers laid out like params, out (sums over the S segments)
 *   dx [S*Tc,B,D] out, may be null
 *   state [L,2,B,H] in/out, may be null: per layer h then c; in: state before the first segment
 *         (null: zeros); out: state after the last segment
 *   reserve: rlstm_stream_reserve_bytes(); workspace: rlstm_stream_workspace_bytes(); all DEVICE.
 *   hip_stream carries the dependent chain; hip_stream_b, if not null and different, takes the weight gradients
 *   of every (segment, layer), which then run beside the layers below (ordering by events created and destroyed
 *   inside the call; when the call returns hip_stream waits for everything placed on hip_stream_b).  The results
 *   do not depend on it up to the order of sums inside the products (another product kernel runs beside the
 *   recurrent kernels).
 * Engines and errors as for lstm_fwd / lstm_bwd (the shape seen by the engine is T = Tc).
 */
typedef struct rlstm_stream_desc {
  int32_t L, S, Tc, B, D, H;
  int32_t operand_dtype;  /* as in rlstm_desc */
  int32_t engine;         /* RLSTM_ENGINE_* */
  int32_t batch_groups, bwd_exchange, gemm_variant;   /* tuning, 0 = default */
} rlstm_stream_desc;
RLSTM_API size_t rlstm_stream_reserve_bytes(const rlstm_stream_desc* desc);
RLSTM_API size_t rlstm_stream_workspace_bytes(const rlstm_stream_desc* desc);
RLSTM_API int lstm_stream_fwd_bwd(const rlstm_stream_desc* desc, const float* x, const float* const* params,
                                  const int32_t* seq_lens, const float* dy_top, float* y_top, float* const* grads,
                                  float* dx, float* state, void* reserve, void* workspace, void* hip_stream,
                                  void* hip_stream_b);

/*
 * softmax_ce_fwd_bwd - the frame-wise output layer of the acoustic model (Sec. 6: a softmax
 * output layer over the tied-state classes on top of the BLSTM stack, trained with the
 * cross-entropy criterion, one of the loss layers of Sec. 3.2; the frame error rate is what Table 1
 * reports) and its gradients:
 *   z = y Wo + bo;  p = softmax(z) per frame;  loss = sum over valid frames of -log p[label];
 *   errors = number of valid frames whose largest p (lowest index on ties) is not the label;
 *   dz = p - onehot(label) on valid frames, 0 elsewhere;  dy = dz Wo^T;  dWo = y^T dz;
 *   dbo = column sums of dz.  A frame (t, b) is valid when t < seq_lens[b] (clamped to [0, T])
 *   and 0 <= label < C; batch gradients are sums, as everywhere in this library.
 *   y [T,B,F] in;  Wo [F,C], bo [C] in;  labels [T,B] int32 in;  seq_lens [B] in;
 *   loss (one float), errors (one int32), dy [T,B,F], dWo [F,C], dbo [C] out; all DEVICE.
 *   operand_dtype as in rlstm_desc (the three products).  workspace: rlstm_ce_workspace_bytes()
 *   bytes of DEVICE scratch (logits with the class dimension padded to a multiple of 4, padded
 *   copies of Wo and dWo, partial sums); RLSTM_ESIZE when workspace_bytes is smaller.
 *   All sums are taken in a fixed order: results are bit-reproducible from run to run.
 *
 * rlstm_sgd_momentum_step, rlstm_adam_step - the two update rules the training runs use (Sec. 4.3,
 * Sec. 6), elementwise over n parameters, in place, DEVICE arrays:
 *   SGD with momentum:  v <- momentum v + g;  param <- param - learning_rate v
 *   Adam (Kingma & Ba): m <- b1 m + (1 - b1) g;  v <- b2 v + (1 - b2) g^2;
 *       param <- param - learning_rate (m / (1 - b1^step)) / (sqrt(v / (1 - b2^step)) + epsilon),
 *       step = 1 for the first update.  RLSTM_EDIM for step < 1 or a beta outside [0, 1).
 *   The hyper-parameters are doubles: 1 - beta and the two bias corrections are formed in double
 *   and rounded to float32 once; the elementwise arithmetic is float32.
 */
RLSTM_API size_t rlstm_ce_workspace_bytes(int T, int B, int F, int C);
RLSTM_API int softmax_ce_fwd_bwd(int T, int B, int F, int C, int operand_dtype, const float* y, const float* Wo,
                                 const float* bo, const int32_t* labels, const int32_t* seq_lens, float* loss,
                                 int32_t* errors, float* dy, float* dWo, float* dbo, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);
RLSTM_API int rlstm_sgd_momentum_step(float* param, const float* grad, float* velocity, size_t n, double learning_rate,
                                      double momentum, void* hip_stream);
RLSTM_API int rlstm_adam_step(float* param, const float* grad, float* m, float* v, size_t n, double learning_rate,
                              double beta1, double beta2, double epsilon, int step, void* hip_stream);

/*
 * How the persistent engine lays a stack's recurrent passes out on this device (for reports).
 * out[10] (host): {groups of workgroups (directions * groups of sequences), sequences per group,
 * rows a group's tiles hold, units per workgroup, workgroups per group in the forward kernel,
 * workgroups per group in the backward kernel, padded H of the forward product, units per K
 * quarter of the backward product (two exchanges per step) or its padded H (one exchange), exchanges
 * per step of the backward pass (the bwd_exchange tuning field), form of the recurrent product's operands:
 * 0 fp32 values on the fp32 matrix instructions, 1 values rounded to bf16, 2 fp32 values as three bf16
 * parts each}.  RLSTM_ERESIDENT if the persistent engine cannot hold the shape.
 */
RLSTM_API int rblstm_plan(const rblstm_desc* d, int32_t* out);

/*
 * Measurement aid (not part of the method): times the bare exchange that one hop of the
 * persistent kernels' step chain consists of, without their arithmetic.  `groups` (1..8) groups
 * of `members` workgroups, placed like the recurrent kernels' (one per CU, workgroup index =
 * member * groups + group); per step every workgroup stores `tile_bytes` (multiple of 16) with
 * device-scope stores, waits for their acknowledgement, raises its step flag, waits for the flags
 * of all members of its group and loads the first `read_bytes` (<= members * tile_bytes) of the
 * group's tiles with device-scope loads.  Runs `steps` steps three times on the stream,
 * synchronises, and writes the best time per step in microseconds to *us_per_step (host pointer).
 * workspace: device memory of at least rlstm_exchange_floor_bytes() bytes (0 = bad arguments).
 * Returns RLSTM_ERESIDENT when groups * members exceeds the CUs, RLSTM_EHIP when a bounded wait
 * expired (1 s) or a HIP call failed.
 */
RLSTM_API size_t rlstm_exchange_floor_bytes(int groups, int members, int tile_bytes);
RLSTM_API int rlstm_exchange_floor(int groups, int members, int tile_bytes, int read_bytes, int steps,
                                   void* workspace, size_t workspace_bytes, float* us_per_step, void* hip_stream);



/*
 * Test hook for the failure path of the persistent kernels (not part of the method).  From the
 * next call on, workgroup `mute_workgroup` of every persistent launch withholds its step flags
 * (-1: none does), and every wait between workgroups is bounded by `wait_ticks` ticks of the
 * 100 MHz wall clock (0: the default of 4 s).  With a muted workgroup the others' waits expire,
 * every workgroup leaves its loop, the kernels end normally, the results are invalid and
 * rlstm_last_timeout() reports 1.  rlstm_test_hook(-1, 0) restores normal operation.
 * The scan kernels of the two-dimensional layer obey the same hook: workgroup `mute_workgroup` hands no
 * row to the neighbouring band, whose wait (default 2 s) then expires.
 */
RLSTM_API int rlstm_test_hook(int mute_workgroup, uint64_t wait_ticks);

/*
 * Test hook against races in the exchange between the workgroups of the persistent kernels (not part of the method).
 * From the next call on, workgroup `slow_workgroup` of every persistent launch holds back what it publishes (its part
 * of h_t or d a_t, then its step flag) for `ticks` ticks of the 100 MHz wall clock, every step (-1: none does; ticks
 * at most 100000 = 1 ms, RLSTM_EDIM beyond).  A consumer that did not wait for its producer would read the values of
 * two steps ago: the outputs must have the bits of an undisturbed call, only later.  rlstm_test_delay(-1, 0) restores
 * normal operation.  The hook is process-wide and not synchronised with running calls: set it while no call is in
 * flight.
 */
RLSTM_API int rlstm_test_delay(int slow_workgroup, uint32_t ticks);

/* Which engine RLSTM_ENGINE_AUTO resolves to for this shape on the current
 * device: RLSTM_ENGINE_PERSISTENT or RLSTM_ENGINE_STEPWISE (negative: error). */
RLSTM_API int rlstm_resolve_engine(const rlstm_desc* desc);

/* Static string for an RLSTM_* code. */
RLSTM_API const char* rlstm_strerror(int code);

/* Library version, "major.minor". */
RLSTM_API const char* rlstm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RLSTM_H */
