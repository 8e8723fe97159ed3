// C ABI of librlstm (declared in include/rlstm.h): argument checks, the
// layout of the reserve / workspace buffers, and the order in which the
// matrix products and the recurrent passes of one layer, and of the stacked
// bidirectional network, are enqueued (Sec. 4.2 and Fig. 1 of the RETURNN paper).
#include "../../include/rlstm.h"
#include "rlstm_internal.h"

#include <cmath>
#include <mutex>
#include <vector>

using namespace rlstm;

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
constexpr size_t kFlagBytes = 256;

// tuning fields shared by the descriptors: 0 = library default
bool tuning_ok(int batch_groups, int bwd_exchange, int gemm_variant) {
  return batch_groups >= 0 && batch_groups <= 8 && bwd_exchange >= 0 && bwd_exchange <= 2 && gemm_variant >= 0 && gemm_variant <= 3;
}

int check_desc(const rlstm_desc* d) {
  if (!d) return RLSTM_ENULL;
  if (d->T <= 0 || d->B <= 0 || d->D <= 0 || d->H <= 0) return RLSTM_EDIM;
  if (d->ldx != 0 && d->ldx < d->D) return RLSTM_EDIM;
  if (d->ldy != 0 && d->ldy < d->H) return RLSTM_EDIM;
  if ((long long)d->T * d->B > (1ll << 30) || (long long)d->H * 4 > (1ll << 24)) return RLSTM_EDIM;
  if (d->direction != 1 && d->direction != -1) return RLSTM_EMODE;
  if (d->operand_dtype != 0 && d->operand_dtype != 1) return RLSTM_EMODE;
  if (d->engine < RLSTM_ENGINE_AUTO || d->engine > RLSTM_ENGINE_STEPWISE) return RLSTM_EMODE;
  if (!tuning_ok(d->batch_groups, d->bwd_exchange, d->gemm_variant)) return RLSTM_EMODE;
  return RLSTM_OK;
}
int check_stack_desc(const rblstm_desc* d) {
  if (!d) return RLSTM_ENULL;
  if (d->L <= 0 || d->T <= 0 || d->B <= 0 || d->D <= 0 || d->H <= 0) return RLSTM_EDIM;
  if ((long long)d->T * d->B > (1ll << 30) || (long long)d->H * 4 > (1ll << 24)) return RLSTM_EDIM;
  if (d->operand_dtype != 0 && d->operand_dtype != 1) return RLSTM_EMODE;
  if (d->engine < RLSTM_ENGINE_AUTO || d->engine > RLSTM_ENGINE_STEPWISE) return RLSTM_EMODE;
  if (!tuning_ok(d->batch_groups, d->bwd_exchange, d->gemm_variant)) return RLSTM_EMODE;
  if (d->first_piece < -1 || d->overlap_mode < 0 || d->overlap_mode > 2) return RLSTM_EMODE;
  return RLSTM_OK;
}

// recurrent shape of one layer in one direction
RecShape layer_rec_shape(const rlstm_desc* d) {
  RecShape s{d->T, d->B, d->H, d->ldy ? d->ldy : d->H, 1, d->operand_dtype};
  s.batch_groups = d->batch_groups; s.bwd_exchange = d->bwd_exchange; s.fp32_instructions = d->gemm_variant != 0;
  return s;
}

size_t splitk_floats(int max_m, int H) {
  // room for 16 partial [max_m, 4H] results
  return align_up((size_t)16 * max_m * 4 * H, 64);
}

// resolves the engine; returns RLSTM_ENGINE_PERSISTENT / _STEPWISE or a negative code
int resolve_engine(int engine, const RecShape& s) {
  if (engine == RLSTM_ENGINE_STEPWISE) return RLSTM_ENGINE_STEPWISE;
  DeviceInfo di;
  if (device_info(&di) != hipSuccess) { (void)hipGetLastError(); return RLSTM_EHIP; }
  const bool ok = rec_persistent_supported(s, di.num_cus, di.max_lds);
  if (engine == RLSTM_ENGINE_PERSISTENT) return ok ? RLSTM_ENGINE_PERSISTENT : RLSTM_ERESIDENT;
  return ok ? RLSTM_ENGINE_PERSISTENT : RLSTM_ENGINE_STEPWISE;
}

// ---- optional event timing of the enqueued kernel groups ---------------------
struct ProfRec { int kind, layer, ndir, steps; double flop; hipEvent_t a, b; };
bool g_prof_on = false;
std::vector<ProfRec> g_prof;
std::vector<hipEvent_t> g_prof_pool;

hipEvent_t prof_event() {
  hipEvent_t e = nullptr;
  if (!g_prof_pool.empty()) { e = g_prof_pool.back(); g_prof_pool.pop_back(); return e; }
  if (hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  return e;
}
struct ProfScope {
  hipStream_t st; hipEvent_t b = nullptr; bool on;
  // steps: recurrent steps covered (0 for a matrix product); flop: algorithmic FLOP of the group
  ProfScope(hipStream_t s, int kind, int layer, int ndir, int steps, double flop, bool enabled = true)
      : st(s), on(g_prof_on && enabled) {
    if (!on) return;
    hipEvent_t a = prof_event(); b = prof_event();
    if (!a || !b) { on = false; return; }
    (void)hipEventRecord(a, st);
    g_prof.push_back(ProfRec{kind, layer, ndir, steps, flop, a, b});
  }
  ~ProfScope() { if (on) (void)hipEventRecord(b, st); }
};

inline double gemm_flop(const GemmCall& g) { return 2.0 * g.M * g.N * g.K; }
inline double rec_flop(const RecShape& s, int steps) { return 2.0 * s.B * s.H * 4.0 * s.H * steps * s.ndir; }

int hip_to_code(hipError_t e, int resident_err) {
  if (e == hipSuccess) return RLSTM_OK;
  (void)hipGetLastError();
  return resident_err ? RLSTM_ERESIDENT : RLSTM_EHIP;
}

#define RLSTM_TRY(expr)                                   \
  do {                                                    \
    hipError_t e_ = (expr);                               \
    if (e_ != hipSuccess) return hip_to_code(e_, resident_err); \
  } while (0)

// weight gradients of one direction: dW = X^T dZ, dR = Hprev^T dZ (Hprev = y shifted by one
// processed frame; the h0 term is added separately by the single-layer entry point)
int weight_grads(hipStream_t st, int layer, int T, int B, int Din, int H, int direction,
                 const float* x, int ldx, const float* y, int ldy, const float* dz,
                 float* dW, float* dR, float* skws, size_t skfloats, bool naive, int operand_dtype,
                 bool small_footprint, int variant, bool accumulate = false,
                 const unsigned short* xt16 = nullptr, const unsigned short* yt16 = nullptr, const unsigned short* dzt16 = nullptr) {
  // xt16 [Din, T*B], yt16 [H, T*B] (this direction's rows), dzt16 [4H, T*B]: TRANSPOSED bf16 copies of x, y, dz (frames
  // contiguous, so that both operands of these products over the frames are read along their rows), or null
  int resident_err = 0;
  GemmCall g;
  g.transA = true; g.transB = false;
  g.M = Din; g.N = 4 * H; g.K = T * B;
  g.A = x; g.lda = ldx; g.B = dz; g.ldb = 4 * H; g.C = dW; g.ldc = 4 * H;
  g.splitk_ws = skws; g.splitk_floats = skfloats; g.naive = naive; g.operand_dtype = operand_dtype;
  g.small_footprint = small_footprint; g.accumulate = accumulate; g.variant = variant;
  if (xt16 && dzt16) { g.A16 = xt16; g.lda16 = T * B; g.transA16 = false; g.B16 = dzt16; g.ldb16 = T * B; g.transB16 = true; }
  {
    ProfScope ps(st, 4, layer, 1, 0, gemm_flop(g));
    RLSTM_TRY(gemm(st, g));
  }
  GemmCall r = g;
  r.M = H; r.K = (T - 1) * B;
  r.lda = ldy; r.C = dR;
  r.A16 = nullptr; r.B16 = nullptr;
  if (direction > 0) { r.A = y; r.B = dz + (size_t)B * 4 * H; }
  else               { r.A = y + (size_t)B * ldy; r.B = dz; }
  if (yt16 && dzt16) {
    // a shift by one frame is a shift by B columns of the transposed copies
    r.lda16 = r.ldb16 = T * B; r.transA16 = false; r.transB16 = true;
    if (direction > 0) { r.A16 = yt16; r.B16 = dzt16 + B; }
    else               { r.A16 = yt16 + B; r.B16 = dzt16; }
  }
  {
    ProfScope ps(st, 5, layer, 1, 0, gemm_flop(r));
    RLSTM_TRY(gemm(st, r));
  }
  return RLSTM_OK;
}

struct StackLayout {
  size_t zg[2], c[2], y;     // offsets (floats) inside one layer's block of the reserve
  size_t per_layer;
};
StackLayout stack_layout(const rblstm_desc* d) {
  StackLayout s;
  const size_t tb = (size_t)d->T * d->B;
  size_t off = 0;
  for (int k = 0; k < 2; ++k) { s.zg[k] = off; off += align_up(tb * 4 * d->H, 64); }
  for (int k = 0; k < 2; ++k) { s.c[k] = off; off += align_up(tb * d->H, 64); }
  s.y = off; off += align_up(tb * 2 * d->H, 64);
  s.per_layer = off;
  return s;
}

// bf16 copies of the operands of the stack's matrix products (operand_dtype 1), each in the layout in which the
// product that reads it walks along its rows (the k index contiguous: the product kernel then takes whole 16-byte
// groups of 8 values from memory straight into LDS):
//   xn [T*B, D], yn [T*B, 2H] per layer                  as stored          projection (A)
//   xt [D, T*B], yt [2H, T*B] per layer, dzt [4H, T*B]   transposed         weight gradients (both operands)
//   wt [4H, din] per direction                          transposed         projection (B)
//   dzn [T*B, 8H] = [d a forward | d a backward], wn [din, 8H] = [W forward | W backward]     input gradient
// The last two hold both directions side by side: the gradient w.r.t. the layer's input, the sum of the two
// directions' products over 4H, is then ONE product over 8H (the sum happens in the accumulators; the output is
// written once instead of written, read and written again).
// One conversion kernel writes both copies of an array from one read of it.  They live behind everything else in the
// workspace; offsets in bf16 elements.
struct MirrorLayout { size_t xn, xt, yn, yt, ystride, wn, wt[2], dzn, dzt[2], total; };
bool stack_mirrors(const rblstm_desc* d) {
  // whole 16-byte groups of 8 values along every contiguous dimension, also after a shift by one frame; and enough
  // frames and units that the products take the kernel that reads the copies (256 x 256 tiles over the whole chip)
  return d->operand_dtype == 1 && d->D % 8 == 0 && d->H % 4 == 0 && d->B % 8 == 0 && (long long)d->T * d->B >= 16384 && d->H >= 256;
}
MirrorLayout mirror_layout(const rblstm_desc* d) {
  MirrorLayout m{};
  if (!stack_mirrors(d)) return m;
  const size_t tb = (size_t)d->T * d->B;
  const size_t dmax = d->D > 2 * d->H ? d->D : 2 * d->H;
  size_t o = 0;
  m.xn = o; o += align_up(tb * d->D, 64);
  m.xt = o; o += align_up(tb * d->D, 64);
  m.ystride = align_up(tb * 2 * d->H, 64);
  m.yn = o; o += (size_t)d->L * m.ystride;
  m.yt = o; o += (size_t)d->L * m.ystride;
  m.wn = o; o += align_up(dmax * 8 * d->H, 64);
  for (int k = 0; k < 2; ++k) { m.wt[k] = o; o += align_up(dmax * 4 * d->H, 64); }
  m.dzn = o; o += align_up(tb * 8 * d->H, 64);
  for (int k = 0; k < 2; ++k) { m.dzt[k] = o; o += align_up(tb * 4 * d->H, 64); }
  m.total = o;
  return m;
}
size_t stack_mirror_offset(const rblstm_desc* d);

RecShape stack_rec_shape(const rblstm_desc* d) {
  RecShape s;
  s.T = d->T; s.B = d->B; s.H = d->H; s.ldy = 2 * d->H; s.ndir = 2; s.operand_dtype = d->operand_dtype;
  s.batch_groups = d->batch_groups; s.bwd_exchange = d->bwd_exchange; s.fp32_instructions = d->gemm_variant != 0;
  return s;
}

// bytes of the workspace in front of the bf16 copies: [flag][recurrent scratch][split-K partials][two dy buffers]
size_t stack_mirror_offset(const rblstm_desc* d) {
  const RecShape s = stack_rec_shape(d);
  const int mm = d->D > 2 * d->H ? d->D : 2 * d->H;
  const size_t dy = align_up((size_t)d->T * d->B * 2 * d->H, 64);
  return align_up(kFlagBytes + align_up(rec_workspace_bytes(s), 256) + (splitk_floats(mm, d->H) + 2 * dy) * sizeof(float), 256);
}

// Pipelining of a layer's recurrent pass with the matrix product that feeds it.  The pass over the
// T steps is cut into pieces [b_k, b_k+1); the product for the frames of piece k+1 runs on the
// second stream while the first stream is inside piece k.  Only the product of piece 0 is exposed,
// so the pieces start small and double (the products run two to three times faster per frame than
// the recurrence, so a piece of twice the size is ready in time).
constexpr int kDefaultFirstPiece = 128;   // steps of piece 0 unless the descriptor says otherwise

// Cutting the passes pays only if a matrix-product workgroup fits on a CU next to a workgroup of
// the persistent kernels (LDS); otherwise the products just queue behind the recurrent launches.
// How the products on stream b run beside the recurrent passes on stream a.
//  kShare:  products and recurrent workgroups share CUs, the passes are cut into pieces and fed one piece ahead.
//           Pays when the recurrent kernels leave the matrix cores idle most of a step (small tiles per workgroup:
//           (sequences per group / 16) * (units per workgroup / 4) <= 2) and both footprints fit a CU's LDS.
//           4 x 500 stack, B = 32: 65.3 ms against 69.9 ms serial, although every recurrent step gets slower
//           (5.9 / 9.0 us against 4.85 / 6.4 us alone).
//  kSerial: one after the other on stream a.  81 segments of 250 frames, 3 x 512: 25.9 ms against 28.6 ms shared
//           (three 16-row tiles per workgroup keep the matrix cores busy; products beside them crawl).
// Also measured and dropped: giving the recurrent kernels half of the CUs and the products the other half (both
// asking for more than half of a CU's LDS): 67.6 ms on the 4 x 500 stack; the products at half rate become the
// critical path and the recurrent steps still slow down (5.9 / 8.3 us) through the shared memory system.
enum OverlapMode { kSerial = 0, kShare = 1 };

// requested: the descriptor's overlap_mode (0 chosen per shape, 1 serial, 2 shared; shared falls back to serial where the
// two LDS footprints do not fit one CU)
// *variant: in, the descriptor's gemm_variant; out, the one the call's products use - where the default product kernel
// for fp32 operands (three bf16 parts, 72 KB of LDS) does not fit beside the recurrent workgroups and the kernels on the
// fp32 matrix instructions (33 KB) do, a shared call keeps to those.
OverlapMode overlap_mode(const RecShape& rs, int operand_dtype, bool persistent, bool two_streams, int requested, int* variant) {
  if (!persistent || !two_streams || requested == 1) return kSerial;
  DeviceInfo di;
  if (device_info(&di) != hipSuccess) { (void)hipGetLastError(); return kSerial; }
  int plan[10];
  const size_t rec = persistent_lds_bytes(rs, di.num_cus, di.max_lds);
  bool fits = rec != 0 && rec + gemm_small_lds_bytes(operand_dtype, *variant) <= di.max_lds;
  int v = *variant;
  if (!fits && rec != 0 && operand_dtype == 0 && v == 0 && rec + gemm_small_lds_bytes(0, 3) <= di.max_lds) { fits = true; v = 3; }
  const bool idle_cores = persistent_plan_info(rs, di.num_cus, di.max_lds, plan) && ((plan[2] + 15) / 16) * (plan[3] / 4) <= 2;
  if (!(fits && (idle_cores || requested == 2))) return kSerial;
  *variant = v;
  return kShare;
}

// first_piece: the descriptor's field (0 = default, -1 = passes not cut, otherwise the steps of piece 0)
std::vector<int> piece_bounds(int T, bool pipelined, int first_piece) {
  std::vector<int> b{0};
  const int first = first_piece == 0 ? kDefaultFirstPiece : first_piece;
  if (pipelined && first > 0) {
    for (long long e = first; e < T; e *= 2) b.push_back((int)e);
    if (b.size() > 1 && T - b.back() < first) b.pop_back();
  }
  b.push_back(T);
  return b;
}

// events that order the two streams; destroyed when the call returns (the dependencies they
// expressed stay in the streams)
struct EventList {
  std::vector<hipEvent_t> evs;
  ~EventList() { for (hipEvent_t ev : evs) (void)hipEventDestroy(ev); }
  // work enqueued on `after` from now on starts when everything enqueued on `first` so far is done
  hipError_t order(hipStream_t first, hipStream_t after) {
    if (first == after) return hipSuccess;
    hipEvent_t ev;
    hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e != hipSuccess) return e;
    evs.push_back(ev);
    e = hipEventRecord(ev, first);
    if (e != hipSuccess) return e;
    return hipStreamWaitEvent(after, ev, 0);
  }
};

// sb == sa: everything in order on one stream, passes uncut
int stack_forward(const rblstm_desc* d, const float* x, const float* const* params, const int32_t* seq_lens,
                  float* y_top, float* res, char* ws, hipStream_t sa, hipStream_t sb, bool persistent) {
  int resident_err = 0;
  const StackLayout lay = stack_layout(d);
  const RecShape rs = stack_rec_shape(d);
  unsigned* flag = reinterpret_cast<unsigned*>(ws);
  void* recws = ws + kFlagBytes;
  const int T = d->T, B = d->B, H = d->H;
  int gv = d->gemm_variant;                      // the product kernels of this call (see overlap_mode)
  const OverlapMode mode = overlap_mode(rs, d->operand_dtype, persistent, sb != sa, d->overlap_mode, &gv);
  if (mode == kSerial) sb = sa;
  const bool pipelined = mode != kSerial;
  const std::vector<int> pb = piece_bounds(T, pipelined, d->first_piece);
  const int np = (int)pb.size() - 1;
  EventList evs;
  RLSTM_TRY(clear_flag(sa, flag));
  // bf16 copies of the products' operands: with uncut passes only (everything in order on one stream)
  const bool mirrors = stack_mirrors(d) && persistent && !pipelined;
  const MirrorLayout ml = mirror_layout(d);
  unsigned short* mir = reinterpret_cast<unsigned short*>(ws + stack_mirror_offset(d));
  const size_t tb = (size_t)T * B;
  if (mirrors) RLSTM_TRY(to_bf16_2d(sa, x, (int)tb, d->D, d->D, mir + ml.xn, 0, mir + ml.xt));
  const unsigned short* in16 = mir + ml.xn;
  const float* in = x;
  int din = d->D;
  for (int l = 0; l < d->L; ++l) {
    float* base = res + (size_t)l * lay.per_layer;
    float* yl = (l == d->L - 1) ? y_top : base + lay.y;
    if (mirrors)
      for (int k = 0; k < 2; ++k) RLSTM_TRY(to_bf16_2d(sa, params[6 * l + 3 * k + 0], din, 4 * H, 4 * H, nullptr, 0, mir + ml.wt[k]));
    RecFwdDir dirs[2];
    for (int k = 0; k < 2; ++k)
      dirs[k] = RecFwdDir{base + lay.zg[k], params[6 * l + 3 * k + 1], nullptr, nullptr, yl + (size_t)k * H,
                          base + lay.c[k], nullptr, nullptr, k == 0 ? 1 : -1};
    // the layer's input (the caller's x, or the layer below on stream a) is complete
    RLSTM_TRY(evs.order(sa, sb));
    for (int pc = 0; pc < np; ++pc) {
      const int s0 = pb[pc], s1 = pb[pc + 1];
      // input part of the frames that steps [s0, s1) visit: direction +1 frames [s0, s1), direction -1 frames [T-s1, T-s0)
      for (int k = 0; k < 2; ++k) {
        const size_t f0 = (k == 0) ? (size_t)s0 : (size_t)(T - s1);
        GemmCall g;
        g.M = (s1 - s0) * B; g.N = 4 * H; g.K = din;
        g.A = in + f0 * B * din; g.lda = din; g.B = params[6 * l + 3 * k + 0]; g.ldb = 4 * H;
        g.C = base + lay.zg[k] + f0 * B * 4 * H; g.ldc = 4 * H; g.bias = params[6 * l + 3 * k + 2];
        g.naive = !persistent; g.operand_dtype = d->operand_dtype; g.variant = gv;
        g.small_footprint = mode == kShare && pc > 0;   // the first piece's product runs while the chain waits for it
        if (mirrors) { g.A16 = in16; g.lda16 = din; g.transA16 = false; g.B16 = mir + ml.wt[k]; g.ldb16 = din; g.transB16 = true; }
        ProfScope ps(sb, 0, l, 1, 0, gemm_flop(g));
        RLSTM_TRY(gemm(sb, g));
      }
      RLSTM_TRY(evs.order(sb, sa));
      ProfScope ps(sa, 1, l, 2, s1 - s0, rec_flop(rs, s1 - s0));
      RLSTM_TRY(rec_forward(sa, rs, dirs, seq_lens, recws, flag, persistent, &resident_err, s0, s1));
    }
    if (mirrors) {
      // the layer's output as bf16: the next layer's projection and, in the backward pass, two weight gradients read it
      unsigned short* yn = mir + ml.yn + (size_t)l * ml.ystride;
      RLSTM_TRY(to_bf16_2d(sa, yl, (int)tb, 2 * H, 2 * H, l + 1 < d->L ? yn : nullptr, 0, mir + ml.yt + (size_t)l * ml.ystride));
      in16 = yn;
    }
    in = yl;
    din = 2 * H;
  }
  return RLSTM_OK;
}

// dR += h0^T dz(first processed valid frame of each sequence).  Direction +1 starts every sequence at frame 0
// (a sequence without frames has dz = 0 there), so the term is one small product accumulated into dR; direction -1
// starts each sequence at its own last frame and keeps the gathering kernel.
int h0_term(hipStream_t st, bool persistent, int operand_dtype, int variant, int T, int B, int H, int direction, const float* h0,
            const float* dz, const int32_t* seq_lens, float* dR) {
  int resident_err = 0;
  if (persistent && direction > 0) {
    GemmCall g;
    g.transA = true;
    g.M = H; g.N = 4 * H; g.K = B;
    g.A = h0; g.lda = H; g.B = dz; g.ldb = 4 * H; g.C = dR; g.ldc = 4 * H; g.accumulate = true;
    g.operand_dtype = operand_dtype; g.variant = variant;
    RLSTM_TRY(gemm(st, g));
    return RLSTM_OK;
  }
  RLSTM_TRY(add_h0_outer(st, T, B, H, direction, h0, dz, seq_lens, dR));
  return RLSTM_OK;
}

// Backward half of a training pass over the stack: consumes the reserve a forward pass left.
int stack_backward(const rblstm_desc* d, const float* x, const float* const* params, const int32_t* seq_lens,
                   const float* dy_top, const float* y_top, float* const* grads, float* dx, float* res, char* ws,
                   hipStream_t sa, hipStream_t sb, bool persistent) {
  const RecShape rs = stack_rec_shape(d);
  int gv = d->gemm_variant;                      // the product kernels of this call (see overlap_mode)
  const OverlapMode mode = overlap_mode(rs, d->operand_dtype, persistent, sb != sa, d->overlap_mode, &gv);
  if (mode == kSerial) sb = sa;
  int rc = RLSTM_OK;
  int resident_err = 0;
  const StackLayout lay = stack_layout(d);
  const int T = d->T, B = d->B, H = d->H, L = d->L;
  unsigned* flag = reinterpret_cast<unsigned*>(ws);
  char* recws = ws + kFlagBytes;
  float* skws = reinterpret_cast<float*>(recws + align_up(rec_workspace_bytes(rs), 256));
  const int mm = d->D > 2 * H ? d->D : 2 * H;
  const size_t skfloats = splitk_floats(mm, H);
  const size_t dyfloats = align_up((size_t)T * B * 2 * H, 64);
  float* dybuf[2] = {skws + skfloats, skws + skfloats + dyfloats};

  // Stream a carries the chain of recurrent passes, stream b every matrix product.  The gradient
  // w.r.t. a layer's input is the dy of the layer below: it is produced on stream b in the pieces,
  // and in the frame order, in which that layer's pass back through time consumes it, one piece
  // ahead; the weight gradients follow on stream b and overlap the rest of that pass.
  const bool pipelined = mode != kSerial;
  const std::vector<int> pb = piece_bounds(T, pipelined, d->first_piece);
  const int np = (int)pb.size() - 1;
  EventList evs;
  std::vector<hipEvent_t> ready;       // ready[pc]: dy of piece pc of the layer about to run is complete
  // bf16 copies of the products' operands (see stack_forward, which left x and every layer's y)
  const bool mirrors = stack_mirrors(d) && persistent && !pipelined;
  const MirrorLayout ml = mirror_layout(d);
  unsigned short* mir = reinterpret_cast<unsigned short*>(ws + stack_mirror_offset(d));
  const size_t tb = (size_t)T * B;

  const float* dy = dy_top;
  for (int l = L - 1; l >= 0; --l) {
    float* base = res + (size_t)l * lay.per_layer;
    const float* yl = (l == L - 1) ? y_top : base + lay.y;
    const float* xin = (l == 0) ? x : res + (size_t)(l - 1) * lay.per_layer + lay.y;
    const int din = (l == 0) ? d->D : 2 * H;
    RecBwdDir dirs[2];
    for (int k = 0; k < 2; ++k) {
      dirs[k] = RecBwdDir{base + lay.zg[k], params[6 * l + 3 * k + 1], base + lay.c[k], nullptr,
                          dy + (size_t)k * H, nullptr, nullptr, nullptr, nullptr, grads[6 * l + 3 * k + 2],
                          k == 0 ? 1 : -1};
    }
    for (int pc = 0; pc < np; ++pc) {
      if (!ready.empty()) RLSTM_TRY(hipStreamWaitEvent(sa, ready[pc], 0));
      ProfScope ps(sa, 2, l, 2, pb[pc + 1] - pb[pc], rec_flop(rs, pb[pc + 1] - pb[pc]));
      RLSTM_TRY(rec_backward(sa, rs, dirs, seq_lens, recws, flag, persistent, &resident_err, pb[pc], pb[pc + 1]));
    }
    ready.clear();
    RLSTM_TRY(evs.order(sa, sb));
    float* dxl = (l == 0) ? dx : dybuf[l & 1];
    const unsigned short* yt16 = nullptr; const unsigned short* xt16 = nullptr;
    if (mirrors) {
      // d a of both directions (as stored for the input gradient, transposed for the weight gradients) and W as bf16
      for (int k = 0; k < 2; ++k) {
        RLSTM_TRY(to_bf16_2d(sb, base + lay.zg[k], (int)tb, 4 * H, 4 * H, dxl ? mir + ml.dzn + (size_t)k * 4 * H : nullptr, 8 * H,
                             mir + ml.dzt[k]));
        if (dxl) RLSTM_TRY(to_bf16_2d(sb, params[6 * l + 3 * k + 0], din, 4 * H, 4 * H, mir + ml.wn + (size_t)k * 4 * H, 8 * H, nullptr));
      }
      yt16 = mir + ml.yt + (size_t)l * ml.ystride;
      xt16 = l == 0 ? mir + ml.xt : mir + ml.yt + (size_t)(l - 1) * ml.ystride;
    }

    if (dxl && l > 0 && sb != sa) {
      // columns [0,H) feed direction +1 of the layer below, which visits frames T-1 .. 0;
      // columns [H,2H) feed direction -1, which visits frames 0 .. T-1
      for (int pc = 0; pc < np; ++pc) {
        const int s0 = pb[pc], s1 = pb[pc + 1];
        for (int tk = 0; tk < 2; ++tk) {
          const size_t f0 = (tk == 0) ? (size_t)(T - s1) : (size_t)s0;
          for (int k = 0; k < 2; ++k) {
            GemmCall g;
            g.transB = true;
            g.M = (s1 - s0) * B; g.N = H; g.K = 4 * H;
            g.A = base + lay.zg[k] + f0 * B * 4 * H; g.lda = 4 * H;
            g.B = params[6 * l + 3 * k + 0] + (size_t)tk * H * 4 * H; g.ldb = 4 * H;
            g.C = dxl + f0 * B * din + (size_t)tk * H; g.ldc = din; g.accumulate = (k == 1);
            g.naive = !persistent; g.operand_dtype = d->operand_dtype; g.variant = gv;
            g.small_footprint = mode == kShare && pc > 0;   // the first piece's product runs while the chain waits for it
            // ... and has too few tiles for the chip (128 at 128 steps x 32 sequences x 500 units): K is split as well
            if (pc == 0) { g.splitk_ws = skws; g.splitk_floats = skfloats; }
            ProfScope ps(sb, 3, l, 1, 0, gemm_flop(g));
            RLSTM_TRY(gemm(sb, g));
          }
        }
        hipEvent_t ev;
        RLSTM_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        evs.evs.push_back(ev);
        RLSTM_TRY(hipEventRecord(ev, sb));
        ready.push_back(ev);
      }
    } else if (dxl && mirrors) {
      // both directions in one product over 8H (see MirrorLayout); A and B name direction +1's fp32 arrays only for
      // the fallback test inside gemm(), which the copies' shapes pass whenever mirrors is set
      GemmCall g;
      g.transB = true;
      g.M = T * B; g.N = din; g.K = 8 * H;
      g.C = dxl; g.ldc = din;
      g.operand_dtype = d->operand_dtype; g.variant = gv;
      g.A16 = mir + ml.dzn; g.lda16 = 8 * H; g.transA16 = false; g.B16 = mir + ml.wn; g.ldb16 = 8 * H; g.transB16 = true;
      g.require_mem16 = true;
      ProfScope ps(sb, 3, l, 1, 0, gemm_flop(g));
      const hipError_t e = gemm(sb, g);
      if (e == hipErrorInvalidValue) {
        // too few tiles for the kernel that reads the copies (tiny T*B): the two products on the fp32 arrays
        (void)hipGetLastError();
        for (int k = 0; k < 2; ++k) {
          GemmCall f;
          f.transB = true;
          f.M = T * B; f.N = din; f.K = 4 * H;
          f.A = base + lay.zg[k]; f.lda = 4 * H; f.B = params[6 * l + 3 * k + 0]; f.ldb = 4 * H;
          f.C = dxl; f.ldc = din; f.accumulate = (k == 1);
          f.operand_dtype = d->operand_dtype; f.variant = gv;
          RLSTM_TRY(gemm(sb, f));
        }
      } else {
        RLSTM_TRY(e);
      }
    } else if (dxl) {
      for (int k = 0; k < 2; ++k) {
        GemmCall g;
        g.transB = true;
        g.M = T * B; g.N = din; g.K = 4 * H;
        g.A = base + lay.zg[k]; g.lda = 4 * H; g.B = params[6 * l + 3 * k + 0]; g.ldb = 4 * H;
        g.C = dxl; g.ldc = din; g.accumulate = (k == 1);
        g.naive = !persistent; g.operand_dtype = d->operand_dtype; g.variant = gv;
        ProfScope ps(sb, 3, l, 1, 0, gemm_flop(g));
        RLSTM_TRY(gemm(sb, g));
      }
      // one stream: already in order
    }
    for (int k = 0; k < 2; ++k) {
      rc = weight_grads(sb, l, T, B, din, H, k == 0 ? 1 : -1, xin, din, yl + (size_t)k * H, 2 * H,
                        base + lay.zg[k], grads[6 * l + 3 * k + 0], grads[6 * l + 3 * k + 1], skws, skfloats,
                        !persistent, d->operand_dtype, mode == kShare && l > 0,     // layer 0's run after the last recurrent piece: nothing beside them
                        gv, false, xt16, yt16 ? yt16 + (size_t)k * H * tb : nullptr, mirrors ? mir + ml.dzt[k] : nullptr);
      if (rc != RLSTM_OK) return rc;
    }
    dy = dxl;
  }
  // the caller's stream a sees the end of everything
  RLSTM_TRY(evs.order(sb, sa));
  return RLSTM_OK;
}

}  // namespace

extern "C" {

const char* rlstm_version(void) { return "0.3"; }

const char* rlstm_strerror(int code) {
  switch (code) {
    case RLSTM_OK: return "success";
    case RLSTM_ENULL: return "a required pointer is null";
    case RLSTM_EDIM: return "a dimension is not positive or a leading dimension is too small";
    case RLSTM_EMODE: return "unsupported direction, operand_dtype or engine";
    case RLSTM_ESIZE: return "buffer too small";
    case RLSTM_ERESIDENT: return "the persistent recurrent kernel cannot hold this shape on this device";
    case RLSTM_EHIP: return "a HIP runtime call failed";
    default: return "unknown rlstm error code";
  }
}

size_t rlstm_reserve_bytes(const rlstm_desc* d) {
  if (check_desc(d) != RLSTM_OK) return 0;
  return align_up((size_t)d->T * d->B * 4 * d->H * sizeof(float), 256);
}

size_t rlstm_workspace_bytes(const rlstm_desc* d) {
  if (check_desc(d) != RLSTM_OK) return 0;
  const RecShape s = layer_rec_shape(d);
  const int mm = d->D > d->H ? d->D : d->H;
  return kFlagBytes + align_up(rec_workspace_bytes(s), 256) + splitk_floats(mm, d->H) * sizeof(float);
}

size_t rblstm_reserve_bytes(const rblstm_desc* d) {
  if (check_stack_desc(d) != RLSTM_OK) return 0;
  // the top layer's output is the caller's y_top: its block ends before the y slot (the last one of a block)
  const StackLayout lay = stack_layout(d);
  return (lay.per_layer * (size_t)(d->L - 1) + lay.y) * sizeof(float);
}

size_t rblstm_workspace_bytes(const rblstm_desc* d) {
  if (check_stack_desc(d) != RLSTM_OK) return 0;
  return stack_mirror_offset(d) + mirror_layout(d).total * sizeof(unsigned short);
}

int rlstm_resolve_engine(const rlstm_desc* d) {
  int rc = check_desc(d);
  if (rc != RLSTM_OK) return rc;
  return resolve_engine(d->engine, layer_rec_shape(d));
}

int rlstm_last_timeout(const void* workspace) {
  if (!workspace) return RLSTM_ENULL;
  if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); return RLSTM_EHIP; }
  unsigned v = 0;
  if (hipMemcpy(&v, workspace, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) { (void)hipGetLastError(); return RLSTM_EHIP; }
  return v != 0 ? 1 : 0;
}

static int static_scratch_address(void** out);

int rlstm_last_timeout_on(const void* workspace, void* hip_stream) {
  if (!workspace) {                               // the scratch of lstm_fwd_noalloc on the current device
    void* ptr = nullptr;
    const int rc = static_scratch_address(&ptr);
    if (rc != RLSTM_OK) return rc;
    workspace = ptr;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  unsigned v = 0;
  if (hipMemcpyAsync(&v, workspace, sizeof(v), hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess) { (void)hipGetLastError(); return RLSTM_EHIP; }
  return v != 0 ? 1 : 0;
}

int rblstm_plan(const rblstm_desc* d, int32_t* out) {
  int rc = check_stack_desc(d);
  if (rc != RLSTM_OK) return rc;
  if (!out) return RLSTM_ENULL;
  DeviceInfo di;
  if (device_info(&di) != hipSuccess) { (void)hipGetLastError(); return RLSTM_EHIP; }
  int v[10];
  if (!persistent_plan_info(stack_rec_shape(d), di.num_cus, di.max_lds, v)) return RLSTM_ERESIDENT;
  for (int i = 0; i < 10; ++i) out[i] = v[i];
  return RLSTM_OK;
}

size_t rlstm_exchange_floor_bytes(int groups, int members, int tile_bytes) {
  if (groups < 1 || groups > 8 || members < 1 || members > 1024 || tile_bytes < 16 || tile_bytes > (1 << 20) || tile_bytes % 16) return 0;
  return exchange_probe_bytes(groups, members, tile_bytes);
}

int rlstm_exchange_floor(int groups, int members, int tile_bytes, int read_bytes, int steps,
                         void* workspace, size_t workspace_bytes, float* us_per_step, void* hip_stream) {
  if (!workspace || !us_per_step) return RLSTM_ENULL;
  const size_t need = rlstm_exchange_floor_bytes(groups, members, tile_bytes);
  if (need == 0 || steps < 1 || steps > 1000000 || read_bytes < 0 || (long long)read_bytes > (long long)members * tile_bytes) return RLSTM_EDIM;
  if (workspace_bytes < need) return RLSTM_ESIZE;
  int resident_err = 0, timed_out = 0;
  RLSTM_TRY(exchange_probe(static_cast<hipStream_t>(hip_stream), groups, members, tile_bytes, read_bytes, steps,
                           workspace, us_per_step, &timed_out, &resident_err));
  return timed_out ? RLSTM_EHIP : RLSTM_OK;
}

int rlstm_test_delay(int slow_workgroup, uint32_t ticks) {
  if (ticks > 100000u) return RLSTM_EDIM;          // at most 1 ms per step
  persistent_test_delay(slow_workgroup, ticks);
  return RLSTM_OK;
}

int rlstm_test_hook(int mute_workgroup, uint64_t wait_ticks) {
  persistent_test_hook(mute_workgroup, wait_ticks);
  mdlstm_test_hook(mute_workgroup, wait_ticks);
  return RLSTM_OK;
}

// ---- two-dimensional LSTM layer ------------------------------------------------
static int check_md_desc(const rmdlstm_desc* d) {
  if (!d) return RLSTM_ENULL;
  if (d->Hh <= 0 || d->Ww <= 0 || d->B <= 0 || d->D <= 0 || d->H <= 0) return RLSTM_EDIM;
  if ((long long)d->Hh * d->Ww * d->B > (1ll << 28)) return RLSTM_EDIM;
  if (d->operand_dtype != 0) return RLSTM_EMODE;
  if (d->engine < RLSTM_ENGINE_AUTO || d->engine > RLSTM_ENGINE_STEPWISE) return RLSTM_EMODE;
  MdShape s{d->Hh, d->Ww, d->B, d->H};
  if (d->engine == RLSTM_ENGINE_PERSISTENT && !mdlstm_supported(s)) return RLSTM_ERESIDENT;
  return RLSTM_OK;
}
// the scan kernels (one launch, bands of rows handing rows on) where the shape fits them, else one launch per anti-diagonal
static bool md_stepwise(const rmdlstm_desc* d) {
  MdShape s{d->Hh, d->Ww, d->B, d->H};
  return d->engine == RLSTM_ENGINE_STEPWISE || (d->engine == RLSTM_ENGINE_AUTO && !mdlstm_supported(s));
}
static size_t md_pixels(const rmdlstm_desc* d) { return (size_t)d->Hh * d->Ww * d->B; }
// For a narrow input x is kept next to [h_up | h_left] so that one product yields dR_u, dR_v and dW.
static bool md_fused(const rmdlstm_desc* d) { return d->D <= 32; }
static int md_stride(const rmdlstm_desc* d) { return (int)align_up((size_t)2 * d->H + (md_fused(d) ? d->D : 0), 4); }
static size_t md_dir_floats(const rmdlstm_desc* d) { return align_up(md_pixels(d) * (6 * d->H + md_stride(d)), 64); }
static int md_grad_rows(const rmdlstm_desc* d) { return md_fused(d) ? md_stride(d) : (d->D > d->H ? d->D : d->H); }
static size_t md_splitk_floats(const rmdlstm_desc* d) {
  // the weight gradients are tiny matrices summed over every pixel: room for 512 partial results
  return align_up((size_t)512 * md_grad_rows(d) * 5 * d->H, 64);
}
static size_t md_stacked_floats(const rmdlstm_desc* d) { return align_up((size_t)4 * md_stride(d) * 5 * d->H, 64); }
// behind the split-K partials: the scan kernels' per-band bias gradients, or the stepwise engine's [P, H] scratch arrays
static size_t md_dbpart_floats(const rmdlstm_desc* d) {
  MdShape s{d->Hh, d->Ww, d->B, d->H, 0};
  return align_up(md_stepwise(d) ? mdlstm_stepwise_scratch_floats(s) : mdlstm_dbpart_floats(s), 64);
}
static size_t md_halo_bytes(const rmdlstm_desc* d) {
  if (md_stepwise(d)) return 0;
  MdShape s{d->Hh, d->Ww, d->B, d->H, 0};
  return align_up(mdlstm_halo_words(s) * sizeof(unsigned long long), 256);
}
static void md_dirs(const rmdlstm_desc* d, float* res, const float* const* params, MdDir* dirs) {
  const size_t P = md_pixels(d);
  for (int k = 0; k < 4; ++k) {
    float* base = res + (size_t)k * md_dir_floats(d);
    dirs[k] = MdDir{base, base + P * 5 * d->H, base + P * 6 * d->H, params[4 * k + 1], params[4 * k + 2]};   // zg | c | hc
  }
}

size_t rmdlstm_reserve_bytes(const rmdlstm_desc* d) {
  if (check_md_desc(d) != RLSTM_OK) return 0;
  return 4 * md_dir_floats(d) * sizeof(float);
}

size_t rmdlstm_workspace_bytes(const rmdlstm_desc* d) {
  if (check_md_desc(d) != RLSTM_OK) return 0;
  // [timeout flag][split-K partials][bias gradients of the bands][stacked weight gradients][rows handed between bands]
  return kFlagBytes + (md_splitk_floats(d) + md_dbpart_floats(d) + md_stacked_floats(d)) * sizeof(float) + md_halo_bytes(d);
}

int mdlstm_fwd(const rmdlstm_desc* d, const float* x, const float* const* params, const int32_t* widths,
               float* y, void* reserve, void* workspace, void* hip_stream) {
  int rc = check_md_desc(d);
  if (rc != RLSTM_OK) return rc;
  if (!x || !params || !widths || !y || !reserve || !workspace) return RLSTM_ENULL;
  for (int i = 0; i < 16; ++i) if (!params[i]) return RLSTM_ENULL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int resident_err = 0;
  const int P = (int)md_pixels(d), H = d->H;
  MdDir dirs[4];
  md_dirs(d, static_cast<float*>(reserve), params, dirs);
  // One input value per pixel (grayscale images): b + x W is an outer product, formed inside the scan kernel
  // instead of being written to and read back from HBM; the kernel also leaves x next to [h_up | h_left].
  const bool stepwise = md_stepwise(d);
  const bool xin = d->D == 1 && !stepwise;
  for (int k = 0; k < 4 && !xin; ++k) {
    GemmCall g;
    g.M = P; g.N = 5 * H; g.K = d->D;
    g.A = x; g.lda = d->D; g.B = params[4 * k + 0]; g.ldb = 5 * H; g.C = dirs[k].zg; g.ldc = 5 * H;
    g.bias = params[4 * k + 3];
    g.naive = stepwise;
    ProfScope ps(st, 0, 0, 1, 0, gemm_flop(g));
    RLSTM_TRY(gemm(st, g));
  }
  MdShape s{d->Hh, d->Ww, d->B, H, md_stride(d)};
  if (md_fused(d) && !xin) RLSTM_TRY(mdlstm_copy_x(st, s, dirs, x, d->D));
  if (stepwise) {
    RLSTM_TRY(clear_flag(st, reinterpret_cast<unsigned*>(workspace)));     // this engine has no waits; the flag only says so
    ProfScope ps(st, 1, 0, 4, d->Hh + d->Ww - 1, 2.0 * P * 2 * H * 5 * H * 4);
    RLSTM_TRY(mdlstm_stepwise_forward(st, s, dirs, widths, y));
    return RLSTM_OK;
  }
  const float* W1[4]; const float* b1[4];
  for (int k = 0; k < 4; ++k) { W1[k] = params[4 * k + 0]; b1[k] = params[4 * k + 3]; }
  const int diag = d->Hh + d->Ww - 1;
  char* ws = static_cast<char*>(workspace);
  float* wsf = reinterpret_cast<float*>(ws + kFlagBytes);
  unsigned long long* halo = reinterpret_cast<unsigned long long*>(wsf + md_splitk_floats(d) + md_dbpart_floats(d) + md_stacked_floats(d));
  ProfScope ps(st, 1, 0, 4, diag, 2.0 * P * 2 * H * 5 * H * 4);
  RLSTM_TRY(mdlstm_forward(st, s, dirs, widths, y, halo, reinterpret_cast<unsigned*>(ws), xin ? x : nullptr, W1, b1));
  return RLSTM_OK;
}

int mdlstm_bwd(const rmdlstm_desc* d, const float* x, const float* const* params, const int32_t* widths,
               void* reserve, const float* dy, float* dx, float* const* grads, void* workspace, void* hip_stream) {
  int rc = check_md_desc(d);
  if (rc != RLSTM_OK) return rc;
  if (!x || !params || !widths || !reserve || !dy || !grads || !workspace) return RLSTM_ENULL;
  for (int i = 0; i < 16; ++i) if (!params[i] || !grads[i]) return RLSTM_ENULL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int resident_err = 0;
  const int P = (int)md_pixels(d), H = d->H, D = d->D;
  MdDir dirs[4];
  md_dirs(d, static_cast<float*>(reserve), params, dirs);
  MdShape s{d->Hh, d->Ww, d->B, H, md_stride(d)};
  char* ws = static_cast<char*>(workspace);
  float* skws = reinterpret_cast<float*>(ws + kFlagBytes);
  const size_t skfloats = md_splitk_floats(d);
  unsigned long long* halo = reinterpret_cast<unsigned long long*>(skws + skfloats + md_dbpart_floats(d) + md_stacked_floats(d));
  {
    float* db[4] = {grads[3], grads[7], grads[11], grads[15]};
    ProfScope ps(st, 2, 0, 4, d->Hh + d->Ww - 1, 2.0 * P * 2 * H * 5 * H * 4);
    if (md_stepwise(d)) RLSTM_TRY(mdlstm_stepwise_backward(st, s, dirs, widths, dy, skws + skfloats, db));
    else RLSTM_TRY(mdlstm_backward(st, s, dirs, widths, dy, skws + skfloats, db, halo, reinterpret_cast<unsigned*>(ws)));
  }
  float* stacked = skws + skfloats + md_dbpart_floats(d);
  const size_t stacked_one = (size_t)s.S * 5 * H;
  for (int k = 0; k < 4; ++k) {
    GemmCall g;
    g.transA = true;
    g.N = 5 * H; g.K = P;
    g.B = dirs[k].zg; g.ldb = 5 * H; g.ldc = 5 * H;
    g.splitk_ws = skws; g.splitk_floats = skfloats;
    if (md_fused(d)) {
      // [h_up | h_left | x]^T dA: d R_u, d R_v and d W stacked.  All S columns of the array take part (S is the
      // row stride, a multiple of 4, which keeps the product on the float4 path); the rows of the result that
      // belong to the padding columns are never read.
      g.M = s.S; g.A = dirs[k].hc; g.lda = s.S; g.C = stacked + (size_t)k * stacked_one;
      ProfScope ps(st, 5, 0, 1, 0, gemm_flop(g));
      RLSTM_TRY(gemm(st, g));
    } else {
      g.M = D; g.A = x; g.lda = D; g.C = grads[4 * k + 0];
      {
        ProfScope ps(st, 4, 0, 1, 0, gemm_flop(g));
        RLSTM_TRY(gemm(st, g));
      }
      for (int w = 0; w < 2; ++w) {      // d R_u from the vertical predecessors' h, d R_v from the horizontal ones'
        GemmCall r = g;
        r.M = H; r.A = dirs[k].hc + (size_t)w * H; r.lda = s.S; r.C = grads[4 * k + 1 + w];
        ProfScope ps(st, 5, 0, 1, 0, gemm_flop(r));
        RLSTM_TRY(gemm(st, r));
      }
    }
    if (dx) {
      GemmCall q;
      q.transB = true;
      q.M = P; q.N = D; q.K = 5 * H;
      q.A = dirs[k].zg; q.lda = 5 * H; q.B = params[4 * k + 0]; q.ldb = 5 * H; q.C = dx; q.ldc = D;
      q.accumulate = k > 0;
      ProfScope ps(st, 3, 0, 1, 0, gemm_flop(q));
      RLSTM_TRY(gemm(st, q));
    }
  }
  if (md_fused(d)) {
    const float* src[4]; float* dRu[4]; float* dRv[4]; float* dWp[4];
    for (int k = 0; k < 4; ++k) {
      src[k] = stacked + (size_t)k * stacked_one;
      dWp[k] = grads[4 * k + 0]; dRu[k] = grads[4 * k + 1]; dRv[k] = grads[4 * k + 2];
    }
    RLSTM_TRY(mdlstm_scatter_grads(st, D, H, src, dRu, dRv, dWp));
  }
  return RLSTM_OK;
}

long long rlstm_chunk_plan(const int32_t* seq_lens, int B, int size, int step, int32_t* chunk_seq, int32_t* chunk_start,
                           int32_t* chunk_len, long long max_chunks) {
  if (!seq_lens) return RLSTM_ENULL;
  if (B <= 0 || size <= 0 || step <= 0 || max_chunks < 0) return RLSTM_EDIM;
  return chunk_plan(seq_lens, B, size, step, chunk_seq, chunk_start, chunk_len, max_chunks);
}

int rlstm_chunk_gather(const float* x, int T, int B, int D, int ldx, const int32_t* chunk_seq, const int32_t* chunk_start,
                       const int32_t* chunk_len, int n_chunks, int size, float* xc, void* hip_stream) {
  if (!x || !chunk_seq || !chunk_start || !chunk_len || !xc) return RLSTM_ENULL;
  if (T <= 0 || B <= 0 || D <= 0 || n_chunks < 0 || size <= 0 || (ldx != 0 && ldx < D)) return RLSTM_EDIM;
  int resident_err = 0;
  RLSTM_TRY(chunk_gather(static_cast<hipStream_t>(hip_stream), x, T, B, D, ldx ? ldx : D, chunk_seq, chunk_start,
                         chunk_len, n_chunks, size, xc));
  return RLSTM_OK;
}

// ---- output layer and parameter updates ------------------------------------------------------
static int ce_pitch(int C) { return (int)align_up((size_t)C, 4); }
static const int kCeSlices = 16;
struct CeLayout { size_t z, wo, dwo, bo, scratch, splitk, total; };
static CeLayout ce_layout(int T, int B, int F, int C) {
  const size_t rows = (size_t)T * B, Cp = ce_pitch(C);
  CeLayout l;
  size_t o = 0;
  l.z = o;       o += align_up(rows * Cp, 64);
  l.wo = o;      o += align_up((size_t)F * Cp, 64);
  l.dwo = o;     o += align_up((size_t)F * Cp, 64);
  l.bo = o;      o += align_up(Cp, 64);
  l.scratch = o; o += align_up(ce_scratch_floats((int)rows, (int)Cp), 64);
  l.splitk = o;  o += align_up((size_t)kCeSlices * F * Cp, 64);
  l.total = o;
  return l;
}

size_t rlstm_ce_workspace_bytes(int T, int B, int F, int C) {
  if (T <= 0 || B <= 0 || F <= 0 || C <= 0 || (long long)T * B > (1ll << 30) / 4) return 0;
  return ce_layout(T, B, F, C).total * sizeof(float);
}

int softmax_ce_fwd_bwd(int T, int B, int F, int C, int operand_dtype, const float* y, const float* Wo, const float* bo,
                       const int32_t* labels, const int32_t* seq_lens, float* loss, int32_t* errors,
                       float* dy, float* dWo, float* dbo, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (T <= 0 || B <= 0 || F <= 0 || C <= 0 || (long long)T * B > (1ll << 30) / 4) return RLSTM_EDIM;
  if (operand_dtype != 0 && operand_dtype != 1) return RLSTM_EMODE;
  if (!y || !Wo || !bo || !labels || !seq_lens || !loss || !errors || !dy || !dWo || !dbo || !workspace) return RLSTM_ENULL;
  const CeLayout lay = ce_layout(T, B, F, C);
  if (workspace_bytes < lay.total * sizeof(float)) return RLSTM_ESIZE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* ws = static_cast<float*>(workspace);
  const int rows = T * B, Cp = ce_pitch(C);
  int resident_err = 0;
  // the class dimension is padded to whole float4s inside the workspace (zero weights, zero gradients there)
  RLSTM_TRY(repitch(st, Wo, C, C, ws + lay.wo, Cp, Cp, F));
  RLSTM_TRY(repitch(st, bo, C, C, ws + lay.bo, Cp, Cp, 1));
  {
    GemmCall g;                                   // logits = y Wo + bo
    g.M = rows; g.N = Cp; g.K = F; g.A = y; g.lda = F; g.B = ws + lay.wo; g.ldb = Cp; g.C = ws + lay.z; g.ldc = Cp;
    g.bias = ws + lay.bo; g.operand_dtype = operand_dtype;
    ProfScope ps(st, 6, 0, 1, 0, gemm_flop(g));
    RLSTM_TRY(gemm(st, g));
  }
  {
    ProfScope ps(st, 7, 0, 1, 0, 0.0);
    RLSTM_TRY(softmax_ce_rows(st, ws + lay.z, Cp, labels, seq_lens, T, B, C, ws + lay.scratch, loss, errors, dbo));
  }
  {
    GemmCall g;                                   // dy = dz Wo^T
    g.transB = true;
    g.M = rows; g.N = F; g.K = Cp; g.A = ws + lay.z; g.lda = Cp; g.B = ws + lay.wo; g.ldb = Cp; g.C = dy; g.ldc = F;
    g.operand_dtype = operand_dtype;
    ProfScope ps(st, 6, 0, 1, 0, gemm_flop(g));
    RLSTM_TRY(gemm(st, g));
  }
  {
    GemmCall g;                                   // dWo = y^T dz
    g.transA = true;
    g.M = F; g.N = Cp; g.K = rows; g.A = y; g.lda = F; g.B = ws + lay.z; g.ldb = Cp; g.C = ws + lay.dwo; g.ldc = Cp;
    g.splitk_ws = ws + lay.splitk; g.splitk_floats = (size_t)kCeSlices * F * Cp; g.operand_dtype = operand_dtype;
    ProfScope ps(st, 6, 0, 1, 0, gemm_flop(g));
    RLSTM_TRY(gemm(st, g));
  }
  RLSTM_TRY(repitch(st, ws + lay.dwo, Cp, Cp, dWo, C, C, F));
  return RLSTM_OK;
}

int rlstm_sgd_momentum_step(float* param, const float* grad, float* velocity, size_t n, double learning_rate, double momentum,
                            void* hip_stream) {
  if (n == 0) return RLSTM_OK;
  if (!param || !grad || !velocity) return RLSTM_ENULL;
  int resident_err = 0;
  RLSTM_TRY(sgd_momentum(static_cast<hipStream_t>(hip_stream), param, grad, velocity, n, (float)learning_rate, (float)momentum));
  return RLSTM_OK;
}

int rlstm_adam_step(float* param, const float* grad, float* m, float* v, size_t n, double learning_rate, double beta1,
                    double beta2, double epsilon, int step, void* hip_stream) {
  if (n == 0) return RLSTM_OK;
  if (!param || !grad || !m || !v) return RLSTM_ENULL;
  if (step < 1 || !(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0)) return RLSTM_EDIM;
  int resident_err = 0;
  RLSTM_TRY(adam(static_cast<hipStream_t>(hip_stream), param, grad, m, v, n, learning_rate, beta1, beta2, epsilon, step));
  return RLSTM_OK;
}

// ---- streaming mode: segments chained by their final states, truncated back-propagation ------------
static int check_stream_desc(const rlstm_stream_desc* d) {
  if (!d) return RLSTM_ENULL;
  if (d->L <= 0 || d->S <= 0 || d->Tc <= 0 || d->B <= 0 || d->D <= 0 || d->H <= 0) return RLSTM_EDIM;
  if (d->L > 64 || (long long)d->S * d->Tc * d->B > (1ll << 30) || (long long)d->H * 4 > (1ll << 24)) return RLSTM_EDIM;
  if (d->operand_dtype != 0 && d->operand_dtype != 1) return RLSTM_EMODE;
  if (d->engine < RLSTM_ENGINE_AUTO || d->engine > RLSTM_ENGINE_STEPWISE) return RLSTM_EMODE;
  if (!tuning_ok(d->batch_groups, d->bwd_exchange, d->gemm_variant)) return RLSTM_EMODE;
  return RLSTM_OK;
}
static RecShape stream_rec_shape(const rlstm_stream_desc* d) {
  RecShape s{d->Tc, d->B, d->H, d->H, 1, d->operand_dtype};
  s.batch_groups = d->batch_groups; s.bwd_exchange = d->bwd_exchange; s.fp32_instructions = d->gemm_variant != 0;
  return s;
}
struct StreamLayout {
  size_t zg, c, y, per_layer;                       // reserve, floats, one segment per layer
  size_t rec, splitk, splitk_floats, dy[2], db, lens, state[2], total;   // workspace, bytes
};
static StreamLayout stream_layout(const rlstm_stream_desc* d) {
  StreamLayout l;
  const size_t tb = (size_t)d->Tc * d->B;
  l.zg = 0; l.c = align_up(tb * 4 * d->H, 64); l.y = l.c + align_up(tb * d->H, 64);
  l.per_layer = l.y + align_up(tb * d->H, 64);
  const RecShape rs = stream_rec_shape(d);
  size_t o = kFlagBytes;
  l.rec = o;     o += align_up(rec_workspace_bytes(rs), 256);
  l.splitk_floats = splitk_floats(d->D > d->H ? d->D : d->H, d->H);
  l.splitk = o;  o += align_up(l.splitk_floats * sizeof(float), 256);
  for (int k = 0; k < 2; ++k) { l.dy[k] = o; o += align_up(tb * d->H * sizeof(float), 256); }
  l.db = o;      o += align_up((size_t)4 * d->H * sizeof(float), 256);
  l.lens = o;    o += align_up((size_t)d->S * d->B * sizeof(int32_t), 256);
  for (int k = 0; k < 2; ++k) { l.state[k] = o; o += align_up((size_t)d->L * 2 * d->B * d->H * sizeof(float), 256); }
  l.total = o;
  return l;
}

size_t rlstm_stream_reserve_bytes(const rlstm_stream_desc* d) {
  if (check_stream_desc(d) != RLSTM_OK) return 0;
  return align_up(stream_layout(d).per_layer * d->L * sizeof(float), 256);
}

size_t rlstm_stream_workspace_bytes(const rlstm_stream_desc* d) {
  if (check_stream_desc(d) != RLSTM_OK) return 0;
  return stream_layout(d).total;
}

int lstm_stream_fwd_bwd(const rlstm_stream_desc* d, const float* x, const float* const* params, const int32_t* seq_lens,
                        const float* dy_top, float* y_top, float* const* grads, float* dx, float* state,
                        void* reserve, void* workspace, void* hip_stream, void* hip_stream_b) {
  int rc = check_stream_desc(d);
  if (rc != RLSTM_OK) return rc;
  if (!x || !params || !seq_lens || !dy_top || !y_top || !grads || !reserve || !workspace) return RLSTM_ENULL;
  for (int i = 0; i < 3 * d->L; ++i) if (!params[i] || !grads[i]) return RLSTM_ENULL;
  const int L = d->L, S = d->S, Tc = d->Tc, B = d->B, D = d->D, H = d->H;
  const RecShape rs = stream_rec_shape(d);
  const int eng = resolve_engine(d->engine, rs);
  if (eng < 0) return eng;
  const bool persistent = eng == RLSTM_ENGINE_PERSISTENT;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // Stream b, if given and different, takes the weight gradients of a (segment, layer): nothing of the segment waits
  // for them, so they run beside the passes back through time of the layers below; the next segment's forward pass
  // of a layer waits for them before it overwrites what they read.  Only where a product workgroup fits on a CU
  // beside a workgroup of the persistent kernels (overlap_mode, as for the bidirectional stack).
  int gv = d->gemm_variant;                      // the product kernels of this call (see overlap_mode)
  hipStream_t sw = hip_stream_b ? static_cast<hipStream_t>(hip_stream_b) : st;
  if (sw != st && overlap_mode(rs, d->operand_dtype, persistent, true, 2, &gv) != kShare) sw = st;
  const bool two = sw != st;
  EventList evs;
  std::vector<hipEvent_t> wdone(L, nullptr);   // weight gradients of the previous segment's layer l are done
  const StreamLayout lay = stream_layout(d);
  float* res = static_cast<float*>(reserve);
  char* ws = static_cast<char*>(workspace);
  unsigned* flag = reinterpret_cast<unsigned*>(ws);
  char* recws = ws + lay.rec;
  float* skws = reinterpret_cast<float*>(ws + lay.splitk);
  float* dybuf[2] = {reinterpret_cast<float*>(ws + lay.dy[0]), reinterpret_cast<float*>(ws + lay.dy[1])};
  float* dbtmp = reinterpret_cast<float*>(ws + lay.db);
  int32_t* lens = reinterpret_cast<int32_t*>(ws + lay.lens);
  float* sbuf[2] = {reinterpret_cast<float*>(ws + lay.state[0]), reinterpret_cast<float*>(ws + lay.state[1])};
  const size_t bh = (size_t)B * H, nstate = (size_t)L * 2 * bh, tb = (size_t)Tc * B;
  int resident_err = 0;

  RLSTM_TRY(clear_flag(st, flag));
  RLSTM_TRY(segment_lens(st, seq_lens, B, S, Tc, lens));
  if (state) RLSTM_TRY(accumulate(st, sbuf[0], state, nstate, true));
  else       RLSTM_TRY(fill_f32(st, sbuf[0], nstate, 0.f));

  for (int s = 0; s < S; ++s) {
    const int32_t* slens = lens + (size_t)s * B;
    float* cur = sbuf[s & 1];          // state the segment starts from: [L][h | c][B, H]
    float* nxt = sbuf[(s + 1) & 1];    // state it ends in
    // forward through the layers
    const float* in = x + (size_t)s * tb * D;
    int din = D;
    for (int l = 0; l < L; ++l) {
      float* base = res + (size_t)l * lay.per_layer;
      float* yl = (l == L - 1) ? y_top + (size_t)s * tb * H : base + lay.y;
      if (two) {
        // this layer's gates and output are about to be overwritten: the previous segment's weight gradients of this
        // layer read them (d a, y), those of the layer above read y as their input
        if (wdone[l]) RLSTM_TRY(hipStreamWaitEvent(st, wdone[l], 0));
        if (l + 1 < L && wdone[l + 1]) RLSTM_TRY(hipStreamWaitEvent(st, wdone[l + 1], 0));
      }
      GemmCall g;
      g.M = Tc * B; g.N = 4 * H; g.K = din;
      g.A = in; g.lda = din; g.B = params[3 * l + 0]; g.ldb = 4 * H; g.C = base + lay.zg; g.ldc = 4 * H;
      g.bias = params[3 * l + 2]; g.naive = !persistent; g.operand_dtype = d->operand_dtype; g.variant = gv;
      {
        ProfScope ps(st, 0, l, 1, 0, gemm_flop(g));
        RLSTM_TRY(gemm(st, g));
      }
      RecFwdDir dir{base + lay.zg, params[3 * l + 1], cur + (size_t)(2 * l) * bh, cur + (size_t)(2 * l + 1) * bh, yl,
                    base + lay.c, nxt + (size_t)(2 * l) * bh, nxt + (size_t)(2 * l + 1) * bh, 1};
      {
        ProfScope ps(st, 1, l, 1, Tc, rec_flop(rs, Tc));
        RLSTM_TRY(rec_forward(st, rs, &dir, slens, recws, flag, persistent, &resident_err, 0, Tc));
      }
      in = yl; din = H;
    }
    // backward through the layers; nothing flows into the segment's final state, and nothing is passed back
    const float* dy = dy_top + (size_t)s * tb * H;
    for (int l = L - 1; l >= 0; --l) {
      float* base = res + (size_t)l * lay.per_layer;
      const float* yl = (l == L - 1) ? y_top + (size_t)s * tb * H : base + lay.y;
      const float* xin = (l == 0) ? x + (size_t)s * tb * D : res + (size_t)(l - 1) * lay.per_layer + lay.y;
      const int dl = (l == 0) ? D : H;
      const float* h0 = cur + (size_t)(2 * l) * bh;
      RecBwdDir dir{base + lay.zg, params[3 * l + 1], base + lay.c, cur + (size_t)(2 * l + 1) * bh, dy, nullptr, nullptr,
                    nullptr, nullptr, dbtmp, 1};
      {
        ProfScope ps(st, 2, l, 1, Tc, rec_flop(rs, Tc));
        RLSTM_TRY(rec_backward(st, rs, &dir, slens, recws, flag, persistent, &resident_err, 0, Tc));
      }
      RLSTM_TRY(accumulate(st, grads[3 * l + 2], dbtmp, (size_t)4 * H, s == 0));
      RLSTM_TRY(evs.order(st, sw));                 // d a of this layer is complete
      rc = weight_grads(sw, l, Tc, B, dl, H, 1, xin, dl, yl, H, base + lay.zg, grads[3 * l + 0], grads[3 * l + 1], skws,
                        lay.splitk_floats, !persistent, d->operand_dtype, two && l > 0, gv, s > 0);
      if (rc != RLSTM_OK) return rc;
      rc = h0_term(sw, persistent, d->operand_dtype, gv, Tc, B, H, 1, h0, base + lay.zg, slens, grads[3 * l + 1]);
      if (rc != RLSTM_OK) return rc;
      if (two) {
        hipEvent_t ev;
        RLSTM_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        evs.evs.push_back(ev);
        RLSTM_TRY(hipEventRecord(ev, sw));
        wdone[l] = ev;
      }
      float* dxl = (l == 0) ? (dx ? dx + (size_t)s * tb * D : nullptr) : dybuf[l & 1];
      if (dxl) {
        GemmCall g;
        g.transB = true;
        g.M = Tc * B; g.N = dl; g.K = 4 * H;
        g.A = base + lay.zg; g.lda = 4 * H; g.B = params[3 * l + 0]; g.ldb = 4 * H; g.C = dxl; g.ldc = dl;
        g.naive = !persistent; g.operand_dtype = d->operand_dtype; g.variant = gv;
        ProfScope ps(st, 3, l, 1, 0, gemm_flop(g));
        RLSTM_TRY(gemm(st, g));
      }
      dy = dxl;
    }
  }
  if (state) RLSTM_TRY(accumulate(st, state, sbuf[S & 1], nstate, true));
  RLSTM_TRY(evs.order(sw, st));                     // the caller's stream sees the end of everything
  return RLSTM_OK;
}

int rlstm_copy_f32(float* dst, const float* src, size_t n, void* hip_stream) {
  if (!dst || !src) return RLSTM_ENULL;
  int resident_err = 0;
  RLSTM_TRY(copy_f32(static_cast<hipStream_t>(hip_stream), dst, src, n));
  return RLSTM_OK;
}

int rlstm_profile_enable(int on) {
  g_prof_on = on != 0;
  return RLSTM_OK;
}

int rlstm_profile_read(rlstm_profile_entry* out, int max_entries) {
  const int n = (int)g_prof.size();
  int rc = n;
  for (int i = 0; i < n; ++i) {
    ProfRec& r = g_prof[i];
    float ms = 0.f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) {
      (void)hipGetLastError();
      rc = RLSTM_EHIP;
    }
    if (out && i < max_entries) out[i] = rlstm_profile_entry{r.kind, r.layer, r.ndir, r.steps, ms, 0.f, r.flop};
    g_prof_pool.push_back(r.a);
    g_prof_pool.push_back(r.b);
  }
  g_prof.clear();
  if (!g_prof_on) {
    // timing is off: give the events back to the runtime so that none outlives the caller's use of the library
    for (hipEvent_t ev : g_prof_pool) (void)hipEventDestroy(ev);
    g_prof_pool.clear();
  }
  return rc;
}

static int gemm_entry(int operand_dtype, int trans_a, int trans_b, int M, int N, int K,
                      const float* A, int lda, const float* B, int ldb, float* C, int ldc,
                      const float* bias, int variant, void* splitk_ws, size_t splitk_ws_bytes, void* hip_stream) {
  if (!A || !B || !C) return RLSTM_ENULL;
  if (M <= 0 || N <= 0 || K < 0) return RLSTM_EDIM;
  if (variant < 0 || variant > 3) return RLSTM_EMODE;
  if (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N) || ldc < N) return RLSTM_EDIM;
  int resident_err = 0;
  GemmCall g;
  g.transA = trans_a != 0; g.transB = trans_b != 0;
  g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.bias = bias;
  g.splitk_ws = static_cast<float*>(splitk_ws); g.splitk_floats = splitk_ws ? splitk_ws_bytes / sizeof(float) : 0;
  g.operand_dtype = operand_dtype; g.variant = variant;
  RLSTM_TRY(gemm(static_cast<hipStream_t>(hip_stream), g));
  return RLSTM_OK;
}

int rlstm_gemm_f32(int trans_a, int trans_b, int M, int N, int K,
                   const float* A, int lda, const float* B, int ldb, float* C, int ldc,
                   const float* bias, int variant, void* splitk_ws, size_t splitk_ws_bytes, void* hip_stream) {
  return gemm_entry(0, trans_a, trans_b, M, N, K, A, lda, B, ldb, C, ldc, bias, variant, splitk_ws, splitk_ws_bytes, hip_stream);
}

int rlstm_gemm_bf16(int trans_a, int trans_b, int M, int N, int K,
                    const float* A, int lda, const float* B, int ldb, float* C, int ldc,
                    const float* bias, int variant, void* splitk_ws, size_t splitk_ws_bytes, void* hip_stream) {
  return gemm_entry(1, trans_a, trans_b, M, N, K, A, lda, B, ldb, C, ldc, bias, variant, splitk_ws, splitk_ws_bytes, hip_stream);
}

// timed = false: no timing events are created, whatever rlstm_profile_enable() says (events are
// allocations of the runtime, which the caller of lstm_fwd_noalloc must not trigger)
static int lstm_fwd_impl(const rlstm_desc* d, const float* x, const float* W, const float* R, const float* b,
                         const float* h0, const float* c0, const int32_t* seq_lens,
                         float* y, float* c, float* hT, float* cT, void* reserve, void* workspace, size_t workspace_bytes,
                         void* hip_stream, bool timed) {
  int rc = check_desc(d);
  if (rc != RLSTM_OK) return rc;
  if (!x || !W || !R || !b || !seq_lens || !y || !c || !reserve || !workspace) return RLSTM_ENULL;
  const int ldx = d->ldx ? d->ldx : d->D;
  const RecShape s = layer_rec_shape(d);
  if (workspace_bytes < kFlagBytes + rec_workspace_bytes_fwd(s)) return RLSTM_ESIZE;
  const int eng = resolve_engine(d->engine, s);
  if (eng < 0) return eng;
  const bool persistent = eng == RLSTM_ENGINE_PERSISTENT;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int resident_err = 0;
  char* ws = static_cast<char*>(workspace);
  unsigned* flag = reinterpret_cast<unsigned*>(ws);
  float* zg = static_cast<float*>(reserve);

  RLSTM_TRY(clear_flag(st, flag));
  GemmCall g;
  g.M = d->T * d->B; g.N = 4 * d->H; g.K = d->D;
  g.A = x; g.lda = ldx; g.B = W; g.ldb = 4 * d->H; g.C = zg; g.ldc = 4 * d->H; g.bias = b;
  g.naive = !persistent; g.operand_dtype = d->operand_dtype; g.variant = d->gemm_variant;
  {
    ProfScope ps(st, 0, 0, 1, 0, gemm_flop(g), timed);
    RLSTM_TRY(gemm(st, g));
  }
  RecFwdDir dir{zg, R, h0, c0, y, c, hT, cT, d->direction};
  {
    ProfScope ps(st, 1, 0, 1, d->T, rec_flop(s, d->T), timed);
    RLSTM_TRY(rec_forward(st, s, &dir, seq_lens, ws + kFlagBytes, flag, persistent, &resident_err, 0, d->T));
  }
  return RLSTM_OK;
}

int rlstm_to_bf16(uint16_t* dst, const float* src, size_t n, void* hip_stream) {
  if (!dst || !src) return RLSTM_ENULL;
  if (n % 8 != 0 || (reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u)) return RLSTM_EDIM;
  int resident_err = 0;
  RLSTM_TRY(to_bf16(static_cast<hipStream_t>(hip_stream), src, dst, n));
  return RLSTM_OK;
}

int rlstm_to_bf16_2d(uint16_t* dst, uint16_t* dst_t, const float* src, int R, int C, int ld, void* hip_stream) {
  if (!src || (!dst && !dst_t)) return RLSTM_ENULL;
  if (R < 0 || C < 0 || ld < C) return RLSTM_EDIM;
  int resident_err = 0;
  const hipError_t e = to_bf16_2d(static_cast<hipStream_t>(hip_stream), src, R, C, ld, dst, 0, dst_t);
  if (e == hipErrorInvalidValue) { (void)hipGetLastError(); return RLSTM_EDIM; }
  RLSTM_TRY(e);
  return RLSTM_OK;
}

int rlstm_gemm_bf16_mem(int trans_a, int trans_b, int M, int N, int K,
                        const uint16_t* A16, int lda, const uint16_t* B16, int ldb,
                        float* C, int ldc, const float* bias, int variant, void* splitk_ws, size_t splitk_ws_bytes, void* hip_stream) {
  if (!A16 || !B16 || !C) return RLSTM_ENULL;
  if (variant != 0 && variant != 3 && variant != 4) return RLSTM_EMODE;
  if (M <= 0 || N <= 0 || K < 0) return RLSTM_EDIM;
  if (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N) || ldc < N) return RLSTM_EDIM;
  int resident_err = 0;
  GemmCall g;
  g.transA = g.transA16 = trans_a != 0; g.transB = g.transB16 = trans_b != 0;
  g.M = M; g.N = N; g.K = K; g.C = C; g.ldc = ldc; g.bias = bias;
  g.A16 = A16; g.lda16 = lda; g.B16 = B16; g.ldb16 = ldb; g.require_mem16 = true;
  g.variant = variant == 3 ? kVariantNoWalk : (variant == 4 ? kVariantNoRing : 0);
  g.splitk_ws = static_cast<float*>(splitk_ws); g.splitk_floats = splitk_ws ? splitk_ws_bytes / sizeof(float) : 0;
  g.operand_dtype = 1;
  const hipError_t e = gemm(static_cast<hipStream_t>(hip_stream), g);
  if (e == hipErrorInvalidValue) { (void)hipGetLastError(); return RLSTM_EMODE; }
  RLSTM_TRY(e);
  return RLSTM_OK;
}

int lstm_fwd(const rlstm_desc* d, const float* x, const float* W, const float* R, const float* b,
             const float* h0, const float* c0, const int32_t* seq_lens,
             float* y, float* c, float* hT, float* cT, void* reserve, void* workspace, void* hip_stream) {
  return lstm_fwd_impl(d, x, W, R, b, h0, c0, seq_lens, y, c, hT, cT, reserve, workspace, (size_t)-1, hip_stream, true);
}

// ---- lstm_fwd for callers that cannot allocate ------------------------------------------------
// The scratch of the recurrent pass (timeout flag, step flags, exchange arrays, carried state) lives in a
// file-scope device array instead of a caller-provided workspace.  Every device the library runs on holds its own
// copy of the array at its own address, until the process ends; the address is looked up once per device.  The
// array's name is only a host-side handle: everything below works with the looked-up device address.
constexpr size_t kStaticScratchBytes = RLSTM_NOALLOC_SCRATCH_LIMIT;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_static_scratch[kMaxDevices] = {};
static std::mutex g_static_scratch_mutex;

// device address of `scratch` on the current device (RLSTM_EHIP if the runtime cannot tell)
static int static_scratch_address(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return RLSTM_EHIP; }
  std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
  if (!g_static_scratch[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return RLSTM_EHIP; }
    g_static_scratch[dev] = ptr;
  }
  *out = g_static_scratch[dev];
  return RLSTM_OK;
}

size_t rlstm_noalloc_scratch_bytes(const rlstm_desc* d) {
  if (check_desc(d) != RLSTM_OK) return 0;
  return kFlagBytes + rec_workspace_bytes_fwd(layer_rec_shape(d));
}

int lstm_fwd_noalloc(const rlstm_desc* d, const float* x, const float* W, const float* R, const float* b,
                     const float* h0, const float* c0, const int32_t* seq_lens,
                     float* y, float* c, float* hT, float* cT, void* reserve, void* hip_stream) {
  int rc = check_desc(d);
  if (rc != RLSTM_OK) return rc;
  if (!x || !W || !R || !b || !seq_lens || !y || !c || !reserve) return RLSTM_ENULL;
  if (rlstm_noalloc_scratch_bytes(d) > kStaticScratchBytes) return RLSTM_ESIZE;
  void* ptr = nullptr;
  rc = static_scratch_address(&ptr);
  if (rc != RLSTM_OK) return rc;
  return lstm_fwd_impl(d, x, W, R, b, h0, c0, seq_lens, y, c, hT, cT, reserve, ptr, kStaticScratchBytes, hip_stream, false);
}

int lstm_bwd(const rlstm_desc* d, const float* x, const float* W, const float* R,
             const int32_t* seq_lens, const float* h0, const float* c0,
             const float* y, const float* c, void* reserve,
             const float* dy, const float* dhT, const float* dcT,
             float* dx, float* dW, float* dR, float* db, float* dh0, float* dc0,
             void* workspace, void* hip_stream) {
  int rc = check_desc(d);
  if (rc != RLSTM_OK) return rc;
  if (!x || !W || !R || !seq_lens || !y || !c || !reserve || !dy || !dW || !dR || !db || !workspace) return RLSTM_ENULL;
  const int ldx = d->ldx ? d->ldx : d->D, ldy = d->ldy ? d->ldy : d->H;
  const int T = d->T, B = d->B, D = d->D, H = d->H;
  const RecShape s = layer_rec_shape(d);
  const int eng = resolve_engine(d->engine, s);
  if (eng < 0) return eng;
  const bool persistent = eng == RLSTM_ENGINE_PERSISTENT;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int resident_err = 0;
  char* ws = static_cast<char*>(workspace);
  unsigned* flag = reinterpret_cast<unsigned*>(ws);
  float* zg = static_cast<float*>(reserve);
  char* recws = ws + kFlagBytes;
  float* skws = reinterpret_cast<float*>(recws + align_up(rec_workspace_bytes(s), 256));
  const size_t skfloats = splitk_floats(D > H ? D : H, H);

  // the timeout flag is left as lstm_fwd left it: a forward pass that gave up keeps the backward kernels from
  // running, and one read of the flag after this call tells about both passes
  RecBwdDir dir{zg, R, c, c0, dy, dhT, dcT, dh0, dc0, db, d->direction};
  {
    ProfScope ps(st, 2, 0, 1, T, rec_flop(s, T));
    RLSTM_TRY(rec_backward(st, s, &dir, seq_lens, recws, flag, persistent, &resident_err, 0, T));
  }
  rc = weight_grads(st, 0, T, B, D, H, d->direction, x, ldx, y, ldy, zg, dW, dR, skws, skfloats, !persistent, d->operand_dtype,
                    false, d->gemm_variant);
  if (rc != RLSTM_OK) return rc;
  if (h0) {
    rc = h0_term(st, persistent, d->operand_dtype, d->gemm_variant, T, B, H, d->direction, h0, zg, seq_lens, dR);
    if (rc != RLSTM_OK) return rc;
  }
  if (dx) {
    GemmCall g;
    g.transB = true;
    g.M = T * B; g.N = D; g.K = 4 * H;
    g.A = zg; g.lda = 4 * H; g.B = W; g.ldb = 4 * H; g.C = dx; g.ldc = ldx;
    g.naive = !persistent; g.operand_dtype = d->operand_dtype; g.variant = d->gemm_variant;
    ProfScope ps(st, 3, 0, 1, 0, gemm_flop(g));
    RLSTM_TRY(gemm(st, g));
  }
  return RLSTM_OK;
}

int blstm_stack_fwd(const rblstm_desc* d, const float* x, const float* const* params,
                    const int32_t* seq_lens, float* y_top, void* reserve, void* workspace, void* hip_stream_a) {
  int rc = check_stack_desc(d);
  if (rc != RLSTM_OK) return rc;
  if (!x || !params || !seq_lens || !y_top || !reserve || !workspace) return RLSTM_ENULL;
  for (int i = 0; i < 6 * d->L; ++i) if (!params[i]) return RLSTM_ENULL;
  const int eng = resolve_engine(d->engine, stack_rec_shape(d));
  if (eng < 0) return eng;
  return stack_forward(d, x, params, seq_lens, y_top, static_cast<float*>(reserve), static_cast<char*>(workspace),
                       static_cast<hipStream_t>(hip_stream_a), static_cast<hipStream_t>(hip_stream_a),
                       eng == RLSTM_ENGINE_PERSISTENT);
}

int blstm_stack_fwd_bwd(const rblstm_desc* d, const float* x, const float* const* params,
                        const int32_t* seq_lens, const float* dy_top,
                        float* y_top, float* const* grads, float* dx,
                        void* reserve, void* workspace, void* hip_stream_a, void* hip_stream_b) {
  int rc = check_stack_desc(d);
  if (rc != RLSTM_OK) return rc;
  if (!x || !params || !seq_lens || !dy_top || !y_top || !grads || !reserve || !workspace) return RLSTM_ENULL;
  for (int i = 0; i < 6 * d->L; ++i) if (!params[i] || !grads[i]) return RLSTM_ENULL;
  const RecShape rs = stack_rec_shape(d);
  const int eng = resolve_engine(d->engine, rs);
  if (eng < 0) return eng;
  const bool persistent = eng == RLSTM_ENGINE_PERSISTENT;
  hipStream_t sa = static_cast<hipStream_t>(hip_stream_a);
  hipStream_t sb = static_cast<hipStream_t>(hip_stream_b);
  const bool overlap = sb != nullptr && sb != sa;
  if (!overlap) sb = sa;

  float* res = static_cast<float*>(reserve);
  char* ws = static_cast<char*>(workspace);
  rc = stack_forward(d, x, params, seq_lens, y_top, res, ws, sa, sb, persistent);
  if (rc != RLSTM_OK) return rc;
  return stack_backward(d, x, params, seq_lens, dy_top, y_top, grads, dx, res, ws, sa, sb, persistent);
}

int blstm_stack_bwd(const rblstm_desc* d, const float* x, const float* const* params,
                    const int32_t* seq_lens, const float* dy_top, const float* y_top,
                    float* const* grads, float* dx,
                    void* reserve, void* workspace, void* hip_stream_a, void* hip_stream_b) {
  int rc = check_stack_desc(d);
  if (rc != RLSTM_OK) return rc;
  if (!x || !params || !seq_lens || !dy_top || !y_top || !grads || !reserve || !workspace) return RLSTM_ENULL;
  for (int i = 0; i < 6 * d->L; ++i) if (!params[i] || !grads[i]) return RLSTM_ENULL;
  const RecShape rs = stack_rec_shape(d);
  const int eng = resolve_engine(d->engine, rs);
  if (eng < 0) return eng;
  hipStream_t sa = static_cast<hipStream_t>(hip_stream_a);
  hipStream_t sb = static_cast<hipStream_t>(hip_stream_b);
  if (sb == nullptr) sb = sa;
  return stack_backward(d, x, params, seq_lens, dy_top, y_top, grads, dx, static_cast<float*>(reserve),
                        static_cast<char*>(workspace), sa, sb, eng == RLSTM_ENGINE_PERSISTENT);
}


}  // extern "C"
