// Persistent engine of the recurrent part of the LSTM layer (Sec. 4.2 of the
// RETURNN paper): the forward time loop h_{t-1} R + gating, and the pass back
// through time, each as ONE launch that runs all T steps of up to
// two independent directions.
//
// Forward.  The H units of a direction are dealt out to Gf workgroups, U units
// each (U = 4 or 8).  A workgroup keeps the i, f, o, g columns of its units of
// R in LDS for the whole kernel, keeps c and h of its (sequence, unit) pairs in
// registers, and per step computes h_{t-1}[B x H] * R[:, its 4U columns] on the
// matrix cores (v_mfma_f32_16x16x4_f32; K split over the 4 wavefronts, partial
// tiles summed through LDS in a fixed order), then applies sigmoid / tanh, the
// cell update and the validity mask (Sec. 5) and stores gates, y and c.
//
// Backward.  d h_{t-1} = d a_t R^T has K = 4H.  The workgroups form a PG x 4
// grid: workgroup (p, q) multiplies the q-th quarter of the rows of d a_t with
// the matching rows of R^T (kept in LDS) for the p-th group of 4U units, and
// hands the partial tile to the four workgroups that own those units; each
// owner adds the four partials in a fixed order.  Gate derivatives, d c and
// d b stay in the owner's registers.
//
// Exchange between workgroups (h_t forwards; d a_t and the partial tiles
// backwards) goes through global memory with device-scope (sc1) stores and
// loads only, never through plain cached accesses, and the data is its own
// ready flag:
//   * h_t and d a_t live in four step buffers (index = step mod 4), stored
//     [group of 4 K-rows][sequence][4]: a producer's values form whole 64-byte
//     lines (no partial-line writes from different workgroups), and a consumer
//     lane fetches with one 16-byte device-scope buffer load the four values it
//     feeds to four consecutive MFMA k-steps (256 contiguous bytes per 16
//     lanes); all loads are issued before the first MFMA.  The K index of the
//     MFMA steps is permuted accordingly, and the resident R / R^T rows are
//     stored in LDS in that same order.  A slot that has not been written yet holds a
//     sentinel (one fixed NaN bit pattern); the consumer re-fetches only the
//     16-byte chunks in which it still sees the sentinel.  Each producer, at
//     step s, first waits until its older stores are acknowledged, then puts
//     the sentinel back into its slots of the buffer that will be used at step
//     s+2 (every reader of that buffer's old content is done by then), then
//     stores its values of step s.  No flag, no acknowledgement wait and no
//     device-wide barrier sits in the step's dependency chain.
//   * partial tiles: every value travels as one 64-bit word (value, step tag),
//     double-buffered, so the owners poll the data itself.
// No cache write-back / invalidate happens in the step loop.  All waits are
// bounded: on expiry the kernel raises the timeout flag and every workgroup
// leaves its loop.
#include "rlstm_internal.h"

namespace rlstm {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr unsigned long long kWaitTimeoutTicks = 400000000ull;   // 4 s of the 100 MHz wall clock
constexpr int CG = 16;                  // 16-byte loads in flight per lane
constexpr int kAuxSc1 = 16;             // buffer-load cache policy: device scope

// ---- bounded spinning --------------------------------------------------------
struct Spin {
  unsigned n = 0;
  unsigned long long t0 = 0;
  // call once per unsuccessful poll; true = give up
  __device__ __forceinline__ bool expired(unsigned* err) {
    if ((++n & 1023u) != 0) return false;
    const unsigned long long now = wall_clock64();
    if (t0 == 0) { t0 = now; return false; }
    if (now - t0 > kWaitTimeoutTicks) return true;
    return __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
  }
};

__device__ __forceinline__ void st_dev(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(unsigned* p, unsigned v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned ld_dev(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_stores_acked() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void compiler_fence() { __atomic_signal_fence(__ATOMIC_SEQ_CST); }

// "not written yet" marker of the exchange arrays: a NaN pattern no arithmetic here produces
constexpr unsigned kSentinel = 0xFFF0DEADu;
constexpr int kStepBuffers = 4;

// fast gate functions: v_exp_f32 / v_rcp_f32 (about 1e-6 absolute error)
__device__ __forceinline__ float fsigmoid(float u) { return __builtin_amdgcn_rcpf(1.0f + __expf(-u)); }
__device__ __forceinline__ float ftanh(float u) { return 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(-2.0f * u)) - 1.0f; }

// Exchange layout: [K-row group r][sequence b][4].  Forward: r = unit / 4 and the 4 entries are
// units 4r..4r+3.  Backward: r = unit and the 4 entries are its gates i, f, o, g.
//
// One wavefront's share of a [B x K] * [K x 16*NT] product over row groups row0 .. row0 + 4*nJ.
// Lane (l16, lq) fetches for chunk (J, mt) the 16 bytes of group row0 + 4J + lq, sequence
// mt*16 + l16, and feeds entry i of it to MFMA step (J, i) as A[row l16][k index lq]; the B rows
// of that step are bs[((J*4 + i)*4 + lq)][...] (LDS, row stride ldb floats), i.e. the caller stores
// its resident matrix in this step order.  Chunks that still hold the sentinel are fetched again
// until their producer has written them.  Returns false if the bounded wait expired.
template <int MT, int NT>
__device__ __forceinline__ bool wave_product(const float* xbuf, int xbuf_bytes, int row0, int nJ, const float* bs, int ldb,
                                             floatx4 (&acc)[MT][NT], unsigned* err) {
  constexpr int Bp = 16 * MT;
  const int lane = threadIdx.x & 63, l16 = lane & 15, lq = lane >> 4;
  __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(xbuf), 0, xbuf_bytes, 0x00020000);
  const int nch = nJ * MT;                       // 16-byte chunks per lane
  const int lane_off = ((row0 + lq) * Bp + l16) * 16;
  bool ok = true;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int c0 = 0; c0 < nch; c0 += CG) {
    floatx4 v[CG];
    const int ng = min(nch - c0, CG);
    unsigned pending = (1u << ng) - 1u;          // chunks of this group still to be fetched (wavefront-uniform)
    Spin sp;
    for (;;) {
      // light spin on the first outstanding chunk only, so that waiting costs one 16-byte load per
      // lane and round trip instead of re-reading the whole block
      {
        const int qf = __builtin_ctz(pending);
        const int Jf = (c0 + qf) / MT, mf = (c0 + qf) % MT;
        for (;;) {
          const intx4 w = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane_off + (4 * Jf * Bp + mf * 16) * 16, 0, kAuxSc1);
          const bool unwritten = (unsigned)w[0] == kSentinel || (unsigned)w[1] == kSentinel ||
                                 (unsigned)w[2] == kSentinel || (unsigned)w[3] == kSentinel;
          if (!__any(unwritten)) break;
          if (sp.expired(err)) { ok = false; break; }
        }
        if (!ok) break;
      }
#pragma unroll
      for (int q = 0; q < CG; ++q)
        if ((pending >> q) & 1u) {
          const int J = c0 / MT + q / MT, mt = q % MT;
          v[q] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(
                                                 rsrc, lane_off + (4 * J * Bp + mt * 16) * 16, 0, kAuxSc1));
        }
      unsigned bad = 0;
#pragma unroll
      for (int q = 0; q < CG; ++q) {
        if ((pending >> q) & 1u) {
          const intx4 w = __builtin_bit_cast(intx4, v[q]);
          const bool unwritten = (unsigned)w[0] == kSentinel || (unsigned)w[1] == kSentinel ||
                                 (unsigned)w[2] == kSentinel || (unsigned)w[3] == kSentinel;
          if (__any(unwritten)) bad |= 1u << q;
        }
      }
      pending = bad;
      if (!pending) break;
      if (sp.expired(err)) { ok = false; break; }
    }
#pragma unroll
    for (int q = 0; q < CG; ++q) {
      if (q < ng) {
        const int J = c0 / MT + q / MT;
        const int mt = q % MT;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const float bf = bs[((J * 4 + i) * 4 + lq) * ldb + nt * 16 + l16];
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(v[q][i], bf, acc[mt][nt], 0, 0, 0);
          }
        }
      }
    }
  }
  compiler_fence();
  return ok;
}

// ---------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------
struct PFwdDir {
  float* zg; const float* R; const float* h0; const float* c0;
  float* y; float* c; float* hT; float* cT;
  float* hx;            // kStepBuffers x [Hp/4][Bp][4]
  int direction;
};
struct PFwdParams {
  PFwdDir d[2];
  const int32_t* seq_lens;
  unsigned* err;
  int T, B, H, ldy, Gf, Hp;
};

// Workgroup = 4 compute wavefronts (threads 0..255) + 1 I/O wavefront (threads 256..319).
// The compute wavefronts touch global memory only through the device-scope exchange; the I/O
// wavefront moves the frame's input part from HBM into LDS one step ahead and the frame's
// outputs (gates, y, c) from LDS to HBM one step behind, so HBM latency and store
// acknowledgements never sit in the step's dependency chain.
constexpr int kBlockThreads = 320;

template <int MT, int NT>
__global__ __launch_bounds__(kBlockThreads) void lstm_fwd_persistent_kernel(PFwdParams p) {
  constexpr int U = 4 * NT, NC = 16 * NT;
  constexpr int NE = MT * 16 * U;                // (sequence, unit) pairs of this workgroup (multiple of 64)
  constexpr int EPT = (NE + 255) / 256;          // pairs per compute thread
  constexpr int EPL = NE / 64;                   // pairs per I/O lane
  extern __shared__ __align__(16) float lds[];
  const int dir = blockIdx.x / p.Gf, wg = blockIdx.x % p.Gf;
  const PFwdDir& D = p.d[dir];
  constexpr int Bp = 16 * MT;
  const int T = p.T, B = p.B, H = p.H, Hp = p.Hp;
  const int u0 = wg * U;
  float* Rs = lds;                               // [Hp][NC], rows in MFMA step order (see wave_product)
  float* Red = Rs + (size_t)Hp * NC;             // [4][MT][NT][256]
  float* zin = Red + 4 * MT * NT * 256;          // [2][4][NE]  input part of the frame, per gate
  float* gout = zin + 2 * 4 * NE;                // [2][6][NE]  gates i,f,o,g, y, c of the frame

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wavefront-uniform, kept in a scalar register
  const bool is_io = wave == 4;
  const int lane = tid & 63;

  const int KW = Hp / 4;                         // rows of h per wavefront (multiple of 16)
  // resident slice of R: slice column g*U + uu is column g*H + u0 + uu of R; LDS row
  // w*KW + (J*4 + i)*4 + lq holds row k = w*KW + 16J + 4lq + i of R
  for (int idx = tid; idx < Hp * NC; idx += kBlockThreads) {
    const int row = idx / NC, col = idx % NC;
    const int w = row / KW, r = row % KW;
    const int k = w * KW + (r >> 4) * 16 + (r & 3) * 4 + ((r >> 2) & 3);
    const int g = col / U, u = u0 + col % U;
    Rs[idx] = (k < H && u < H) ? D.R[(size_t)k * 4 * H + g * H + u] : 0.f;
  }
  const size_t hxsz = (size_t)Hp * Bp;           // floats per step buffer

  // compute threads: carried state of the pairs they own
  float hreg[EPT], creg[EPT];
  int eb[EPT], eu[EPT], elen[EPT], eslot[EPT];
  bool ev[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int j = tid + e * 256;
    eb[e] = j / U; eu[e] = u0 + j % U;
    ev[e] = !is_io && (j < NE) && eb[e] < B && eu[e] < H;
    hreg[e] = 0.f; creg[e] = 0.f; elen[e] = 0; eslot[e] = 0;
    if (ev[e]) {
      if (D.h0) hreg[e] = D.h0[(size_t)eb[e] * H + eu[e]];
      if (D.c0) creg[e] = D.c0[(size_t)eb[e] * H + eu[e]];
      elen[e] = min(max(p.seq_lens[eb[e]], 0), T);
      eslot[e] = ((eu[e] >> 2) * Bp + eb[e]) * 4 + (eu[e] & 3);
    }
  }
  // I/O lanes: the pairs they move
  int ib[EPL], iu[EPL];
  bool iv[EPL];
  float zr[EPL][4];
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int j = lane + i * 64;
    ib[i] = j / U; iu[i] = u0 + j % U;
    iv[i] = is_io && ib[i] < B && iu[i] < H;
  }
  auto io_load = [&](int step) {                 // input part of the frame of `step` -> registers
    const int t = D.direction > 0 ? step : T - 1 - step;
#pragma unroll
    for (int i = 0; i < EPL; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        zr[i][g] = iv[i] ? D.zg[((size_t)t * B + ib[i]) * 4 * H + g * H + iu[i]] : 0.f;
  };
  auto io_stage = [&](int step) {                // registers -> LDS buffer of `step`
    float* dst = zin + (step & 1) * 4 * NE;
#pragma unroll
    for (int i = 0; i < EPL; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) dst[g * NE + lane + i * 64] = zr[i][g];
  };
  auto io_store = [&](int step) {                // outputs of the frame of `step`: LDS -> HBM
    const int t = D.direction > 0 ? step : T - 1 - step;
    const float* src = gout + (step & 1) * 6 * NE;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      if (!iv[i]) continue;
      const int j = lane + i * 64;
      const size_t row = (size_t)t * B + ib[i];
      float* zrow = D.zg + row * 4 * H + iu[i];
      zrow[0] = src[0 * NE + j]; zrow[H] = src[1 * NE + j]; zrow[2 * H] = src[2 * NE + j]; zrow[3 * H] = src[3 * NE + j];
      D.y[row * p.ldy + iu[i]] = src[4 * NE + j];
      D.c[row * H + iu[i]] = src[5 * NE + j];
    }
  };
  if (is_io) {
    io_load(0);
    io_stage(0);
    if (T > 1) io_load(1);
  }
  __syncthreads();


  for (int s = 0; s < T; ++s) {
    const int t = D.direction > 0 ? s : T - 1 - s;
    const float* hprev = D.hx + (size_t)((s + 3) & 3) * hxsz;    // h of step s-1
    float* hcur = D.hx + (size_t)(s & 3) * hxsz;
    float* hreset = D.hx + (size_t)((s + 2) & 3) * hxsz;         // holds h of step s-2: nobody reads it any more
    int fail = 0;

    if (!is_io) {
      // h_prev * R over this wavefront's rows of h_prev, fetched as soon as their producers have written them
      floatx4 acc[MT][NT];
      if (!wave_product<MT, NT>(hprev, (int)(hxsz * 4), wave * (KW / 4), KW / 16, Rs + (size_t)wave * KW * NC, NC, acc, p.err))
        fail = 1;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          *reinterpret_cast<floatx4*>(Red + ((wave * MT + mt) * NT + nt) * 256 + lane * 4) = acc[mt][nt];
    } else {
      // stage the next frame's input part (loaded a step ago), write out the previous frame's
      // outputs, start loading the frame after next: every wait here is on work issued a step ago
      if (s + 1 < T) io_stage(s + 1);
      if (s > 0) io_store(s - 1);
      if (s + 2 < T) io_load(s + 2);
    }
    if (__syncthreads_or(fail)) {
      if (tid == 0) st_dev(p.err, 1u);
      return;
    }

    if (!is_io) {
      // gating, cell update, mask; publish the carried h; leave the frame's outputs in LDS
      const float* zcur = zin + (s & 1) * 4 * NE;
      float* ocur = gout + (s & 1) * 6 * NE;
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        if (!ev[e]) continue;
        const int j = tid + e * 256;
        const int b = eb[e], uu = eu[e] - u0;
        const int mt = b >> 4, r = b & 15;
        float a[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int col = g * U + uu;
          const int nt = col >> 4, n = col & 15;
          const int src = ((r >> 2) * 16 + n) * 4 + (r & 3);    // accumulator (row r, col n) of a 16x16 tile
          float sum = zcur[g * NE + j];
#pragma unroll
          for (int w = 0; w < 4; ++w) sum += Red[((w * MT + mt) * NT + nt) * 256 + src];
          a[g] = sum;
        }
        const float gi = fsigmoid(a[0]), gf = fsigmoid(a[1]), go = fsigmoid(a[2]), gg = ftanh(a[3]);
        const float cn = gf * creg[e] + gi * gg;
        const float hn = go * ftanh(cn);
        const bool valid = t < elen[e];
        if (valid) { creg[e] = cn; hreg[e] = hn; }
        ocur[0 * NE + j] = gi; ocur[1 * NE + j] = gf; ocur[2 * NE + j] = go; ocur[3 * NE + j] = gg;
        ocur[4 * NE + j] = valid ? hn : 0.f;
        ocur[5 * NE + j] = creg[e];
      }
      // older stores (issued a step ago) acknowledged -> sentinel into the buffer of step s+2 -> publish h of step s
      wait_stores_acked();
#pragma unroll
      for (int e = 0; e < EPT; ++e)
        if (ev[e]) st_dev(reinterpret_cast<unsigned*>(hreset) + eslot[e], kSentinel);
#pragma unroll
      for (int e = 0; e < EPT; ++e)
        if (ev[e]) st_dev(hcur + eslot[e], hreg[e]);
    }
    __syncthreads();

  }
  __syncthreads();
  if (is_io) io_store(T - 1);

#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    if (!ev[e]) continue;
    if (D.hT) D.hT[(size_t)eb[e] * H + eu[e]] = hreg[e];
    if (D.cT) D.cT[(size_t)eb[e] * H + eu[e]] = creg[e];
  }
}

// ---------------------------------------------------------------------------
// backward
// ---------------------------------------------------------------------------
struct PBwdDir {
  float* zg; const float* R; const float* c; const float* c0; const float* dy;
  const float* dhT; const float* dcT; float* dh0; float* dc0; float* db;
  float* dzx;                   // kStepBuffers x [4*Hq units][Bp][4 gates]
  unsigned long long* part;     // 2 x [PG][4][Bp][UG] (value, tag)
  int direction;
};
struct PBwdParams {
  PBwdDir d[2];
  const int32_t* seq_lens;
  unsigned* err;
  int T, B, H, ldy, PG, Hq;
};

// Same workgroup shape as the forward kernel: 4 compute wavefronts + 1 I/O wavefront that stages
// the frame's gates, cell states and dy from HBM into LDS one step ahead and writes d a back to
// HBM one step behind.
template <int MT, int NT>
__global__ __launch_bounds__(kBlockThreads) void lstm_bwd_persistent_kernel(PBwdParams p) {
  constexpr int U = 4 * NT, UG = 16 * NT, Bp = 16 * MT;
  constexpr int NE = MT * 16 * U;                // (sequence, unit) pairs owned by this workgroup
  constexpr int EPT = (NE + 255) / 256;
  constexpr int EPL = NE / 64;
  extern __shared__ __align__(16) float lds[];
  const int Gb = 4 * p.PG;
  const int dir = blockIdx.x / Gb, wg = blockIdx.x % Gb;
  const int pg = wg >> 2, qq = wg & 3;           // unit group, K quarter (also: which quarter of the group it owns)
  const PBwdDir& D = p.d[dir];
  const int T = p.T, B = p.B, H = p.H, Hq = p.Hq;
  const int u0 = wg * U;                         // owned units
  float* RTs = lds;                              // [4*Hq][UG], rows in MFMA step order (see wave_product)
  float* Red = RTs + (size_t)4 * Hq * UG;        // [4][MT][NT][256]
  float* bin = Red + 4 * MT * NT * 256;          // [2][7][NE]  gates i,f,o,g, c, c_prev, dy of the frame
  float* dzo = bin + 2 * 7 * NE;                 // [2][4][NE]  d a of the frame

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wavefront-uniform, kept in a scalar register
  const bool is_io = wave == 4;
  const int lane = tid & 63;
  const int UW = Hq / 4;                         // units per wavefront of a quarter
  // Quarters that hold no unit (small H) contribute nothing: their workgroups publish no partial
  // tile and owners do not wait for one.  Every workgroup that does publish is paced by the d a
  // of real producers, so no tile is overwritten before its owners have read it.
  const int nq = (H + Hq - 1) / Hq;

  // resident rows of R^T: LDS row w*Hq + (J*4 + g)*4 + lq holds, for unit uk = qq*Hq + w*UW + 4J + lq
  // and gate g, the values R[pg*UG + n][g*H + uk], n = 0..UG-1
  for (int idx = tid; idx < 4 * Hq * UG; idx += kBlockThreads) {
    const int row = idx / UG, n = idx % UG;
    const int w = row / Hq, r = row % Hq;
    const int uk = qq * Hq + w * UW + (r >> 4) * 4 + (r & 3), g = (r >> 2) & 3;
    const int un = pg * UG + n;
    RTs[idx] = (uk < H && un < H) ? D.R[(size_t)un * 4 * H + g * H + uk] : 0.f;
  }
  const size_t xsz = (size_t)16 * Hq * Bp;       // floats per step buffer
  const size_t psz = (size_t)p.PG * 4 * Bp * UG;

  // compute threads: carried gradients of the pairs they own
  float Dh[EPT], Dc[EPT], dbacc[EPT][4];
  int eb[EPT], eu[EPT], elen[EPT], eslot[EPT];
  bool ev[EPT], vprev[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int j = tid + e * 256;
    eb[e] = j / U; eu[e] = u0 + j % U;
    ev[e] = !is_io && (j < NE) && eb[e] < B && eu[e] < H;
    Dh[e] = 0.f; Dc[e] = 0.f; elen[e] = 0; eslot[e] = 0; vprev[e] = false;
#pragma unroll
    for (int g = 0; g < 4; ++g) dbacc[e][g] = 0.f;
    if (ev[e]) {
      if (D.dhT) Dh[e] = D.dhT[(size_t)eb[e] * H + eu[e]];
      if (D.dcT) Dc[e] = D.dcT[(size_t)eb[e] * H + eu[e]];
      elen[e] = min(max(p.seq_lens[eb[e]], 0), T);
      eslot[e] = (eu[e] * Bp + eb[e]) * 4;         // the 4 gates of (unit, sequence) are one 16-byte entry
    }
  }

  // I/O lanes: the pairs they move.  Frames are visited in the reverse of the forward order:
  // step s visits t(s); the frame processed before it in the forward pass is visited at step s+1,
  // so c of step s+1's frame is c_prev of step s's frame.
  int ib[EPL], iu[EPL];
  bool iv[EPL];
  float lr[EPL][6];                              // gates, c_prev, dy in flight
  float cnext[EPL];                              // c of the frame staged next
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int j = lane + i * 64;
    ib[i] = j / U; iu[i] = u0 + j % U;
    iv[i] = is_io && ib[i] < B && iu[i] < H;
    cnext[i] = 0.f;
  }
  auto frame_of = [&](int step) { return D.direction > 0 ? T - 1 - step : step; };
  auto io_load = [&](int step) {
    const int t = frame_of(step);
    const int tprev = D.direction > 0 ? t - 1 : t + 1;     // frame processed before t in the forward pass
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      if (!iv[i]) continue;
      const size_t row = (size_t)t * B + ib[i];
      const float* zrow = D.zg + row * 4 * H + iu[i];
      lr[i][0] = zrow[0]; lr[i][1] = zrow[H]; lr[i][2] = zrow[2 * H]; lr[i][3] = zrow[3 * H];
      if (tprev >= 0 && tprev < T) lr[i][4] = D.c[((size_t)tprev * B + ib[i]) * H + iu[i]];
      else lr[i][4] = D.c0 ? D.c0[(size_t)ib[i] * H + iu[i]] : 0.f;
      lr[i][5] = D.dy[row * p.ldy + iu[i]];
    }
  };
  auto io_stage = [&](int step) {
    float* dst = bin + (step & 1) * 7 * NE;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const int j = lane + i * 64;
#pragma unroll
      for (int g = 0; g < 4; ++g) dst[g * NE + j] = iv[i] ? lr[i][g] : 0.f;
      dst[4 * NE + j] = cnext[i];
      dst[5 * NE + j] = iv[i] ? lr[i][4] : 0.f;
      dst[6 * NE + j] = iv[i] ? lr[i][5] : 0.f;
      cnext[i] = iv[i] ? lr[i][4] : 0.f;
    }
  };
  auto io_store = [&](int step) {
    const int t = frame_of(step);
    const float* src = dzo + (step & 1) * 4 * NE;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      if (!iv[i]) continue;
      const int j = lane + i * 64;
      float* zrow = D.zg + ((size_t)t * B + ib[i]) * 4 * H + iu[i];
      zrow[0] = src[0 * NE + j]; zrow[H] = src[1 * NE + j]; zrow[2 * H] = src[2 * NE + j]; zrow[3 * H] = src[3 * NE + j];
    }
  };
  if (is_io) {
    const int t0 = frame_of(0);
#pragma unroll
    for (int i = 0; i < EPL; ++i)
      if (iv[i]) cnext[i] = D.c[((size_t)t0 * B + ib[i]) * H + iu[i]];
    io_load(0);
    io_stage(0);
    if (T > 1) io_load(1);
  }
  __syncthreads();


  // sums the partial tiles of step `step` for the owned pairs (tag = step + 1)
  auto collect = [&](int step, float (&out)[EPT]) -> int {
    int fail = 0;
    const unsigned long long* pbuf = D.part + (size_t)(step & 1) * psz;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      out[e] = 0.f;
      if (!ev[e]) continue;
      const int n = qq * U + (eu[e] - u0);
      const unsigned long long* src = pbuf + ((size_t)(pg * 4) * Bp + eb[e]) * UG + n;
      unsigned long long v[4];
      Spin sp;
      for (;;) {
        bool ok = true;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          v[k] = 0ull;
          if (k < nq) {
            v[k] = __hip_atomic_load(src + (size_t)k * Bp * UG, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ok = ok && (unsigned)(v[k] >> 32) == (unsigned)(step + 1);
          }
        }
        if (ok) break;
        if (sp.expired(p.err)) { fail = 1; break; }
      }
      float sum = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) sum += __uint_as_float((unsigned)v[k]);
      out[e] = sum;
    }
    return fail;
  };

  for (int s = 0; s < T; ++s) {
    const int t = frame_of(s);
    const float* dzcur = D.dzx + (size_t)(s & 3) * xsz;        // buffer (s+2) mod 4 holds d a of step s-2: nobody reads it any more
    int fail = 0;

    if (!is_io) {
      // d h carried into this frame: product of the previous step (+ carried d h where that frame was invalid)
      if (s > 0) {
        float g[EPT];
        fail = collect(s - 1, g);
#pragma unroll
        for (int e = 0; e < EPT; ++e) Dh[e] = vprev[e] ? g[e] : g[e] + Dh[e];
      }
      // gate derivatives; publish d a of this frame
      const float* in = bin + (s & 1) * 7 * NE;
      float* out = dzo + (s & 1) * 4 * NE;
      float dz[EPT][4];
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        vprev[e] = false;
#pragma unroll
        for (int g = 0; g < 4; ++g) dz[e][g] = 0.f;
        if (!ev[e]) continue;
        const int j = tid + e * 256;
        const bool m = t < elen[e];
        vprev[e] = m;
        if (m) {
          const float gi = in[0 * NE + j], gf = in[1 * NE + j], go = in[2 * NE + j], gg = in[3 * NE + j];
          const float tc = ftanh(in[4 * NE + j]);
          const float dh = in[6 * NE + j] + Dh[e];
          const float d_o = dh * tc;
          const float dc = Dc[e] + dh * go * (1.0f - tc * tc);
          dz[e][0] = dc * gg * gi * (1.0f - gi);
          dz[e][1] = dc * in[5 * NE + j] * gf * (1.0f - gf);
          dz[e][2] = d_o * go * (1.0f - go);
          dz[e][3] = dc * gi * (1.0f - gg * gg);
          Dc[e] = dc * gf;
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          out[g * NE + j] = dz[e][g];
          dbacc[e][g] += dz[e][g];
        }
      }
      // older stores (issued a step ago) acknowledged -> sentinel into the buffer of step s+2 -> publish d a of step s
      wait_stores_acked();
      {
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(D.dzx, 0, (int)(kStepBuffers * xsz * 4), 0x00020000);
        const intx4 sent = intx4{(int)kSentinel, (int)kSentinel, (int)kSentinel, (int)kSentinel};
#pragma unroll
        for (int e = 0; e < EPT; ++e)
          if (ev[e])
            __builtin_amdgcn_raw_buffer_store_b128(sent, rs, (int)((((s + 2) & 3) * xsz + eslot[e]) * 4), 0, kAuxSc1);
#pragma unroll
        for (int e = 0; e < EPT; ++e)
          if (ev[e])
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(intx4, floatx4{dz[e][0], dz[e][1], dz[e][2], dz[e][3]}), rs,
                                                   (int)(((s & 3) * xsz + eslot[e]) * 4), 0, kAuxSc1);
      }
    } else {
      // stage the next frame's inputs (loaded a step ago), write out the previous frame's d a,
      // start loading the frame after next: every wait here is on work issued a step ago
      if (s + 1 < T) io_stage(s + 1);
      if (s > 0) io_store(s - 1);
      if (s + 2 < T) io_load(s + 2);
    }
    if (__syncthreads_or(fail)) {
      if (tid == 0) st_dev(p.err, 1u);
      return;
    }
    // this workgroup's quarter of d a_t R^T for its unit group
    fail = 0;
    if (!is_io && qq < nq) {
      floatx4 acc[MT][NT];
      if (!wave_product<MT, NT>(dzcur, (int)(xsz * 4), qq * Hq + wave * UW, UW / 4, RTs + (size_t)wave * Hq * UG, UG, acc, p.err))
        fail = 1;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          *reinterpret_cast<floatx4*>(Red + ((wave * MT + mt) * NT + nt) * 256 + lane * 4) = acc[mt][nt];
    }
    if (__syncthreads_or(fail)) {
      if (tid == 0) st_dev(p.err, 1u);
      return;
    }
    // sum the four wavefronts' tiles in order and hand (value, tag) to the owners
    if (!is_io && qq < nq) {
      unsigned long long* pbuf = D.part + (size_t)(s & 1) * psz + (size_t)(pg * 4 + qq) * Bp * UG;
      const int ln = tid >> 2, reg = tid & 3;
      const int row = 4 * (ln >> 4) + reg, col = ln & 15;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          float sum = 0.f;
#pragma unroll
          for (int w = 0; w < 4; ++w) sum += Red[((w * MT + mt) * NT + nt) * 256 + tid];
          const unsigned long long word = ((unsigned long long)(unsigned)(s + 1) << 32) | __float_as_uint(sum);
          __hip_atomic_store(pbuf + (size_t)(mt * 16 + row) * UG + nt * 16 + col, word, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // Red is rewritten only after the next step's first workgroup barrier
  }

  // last frame's d a, gradient w.r.t. the initial state, bias gradient of the owned columns
  int fail = 0;
  if (is_io) {
    io_store(T - 1);
  } else {
    float g[EPT];
    fail = collect(T - 1, g);
#pragma unroll
    for (int e = 0; e < EPT; ++e) Dh[e] = vprev[e] ? g[e] : g[e] + Dh[e];
  }
  if (__syncthreads_or(fail)) {
    if (tid == 0) st_dev(p.err, 1u);
    return;
  }
  float* stage = Red;                            // [Bp][4U]
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int j = tid + e * 256;
    if (!is_io && j < NE) {
      const int b = j / U, uu = j % U;
#pragma unroll
      for (int g = 0; g < 4; ++g) stage[b * 4 * U + g * U + uu] = ev[e] ? dbacc[e][g] : 0.f;
    }
    if (!ev[e]) continue;
    if (D.dh0) D.dh0[(size_t)eb[e] * H + eu[e]] = Dh[e];
    if (D.dc0) D.dc0[(size_t)eb[e] * H + eu[e]] = Dc[e];
  }
  __syncthreads();
  if (tid < 4 * U) {
    const int g = tid / U, u = u0 + tid % U;
    if (u < H) {
      float sum = 0.f;
      for (int b = 0; b < B; ++b) sum += stage[b * 4 * U + tid];
      D.db[g * H + u] = sum;
    }
  }
}

// ---------------------------------------------------------------------------
// set-up kernels: clear the exchange arrays and tile tags (padding slots stay 0 for good), then put
// the sentinel into every slot that a producer will write, and h0 where step 0 reads it
// ---------------------------------------------------------------------------
struct PrepParams {
  unsigned* zero_words[2]; size_t nzero[2];       // per direction: words to clear (exchange arrays [+ partial tiles])
  float* xbase[2]; const float* h0[2];            // exchange arrays; forward only: h0 or null
  int ndir, B, H, Bp, backward;
  size_t bufsz;                                   // floats per step buffer
};
__global__ __launch_bounds__(256) void prep_kernel(PrepParams p) {
  const size_t gtid = (size_t)blockIdx.x * 256 + threadIdx.x, gsz = (size_t)gridDim.x * 256;
  for (int d = 0; d < p.ndir; ++d)
    for (size_t i = gtid; i < p.nzero[d]; i += gsz) p.zero_words[d][i] = 0u;
}
__global__ __launch_bounds__(256) void seed_kernel(PrepParams p) {
  const size_t gtid = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (gtid >= (size_t)p.B * p.H) return;
  const int b = (int)(gtid / p.H), u = (int)(gtid % p.H);
  for (int d = 0; d < p.ndir; ++d) {
    unsigned* x = reinterpret_cast<unsigned*>(p.xbase[d]);
    if (!p.backward) {
      const size_t slot = ((size_t)(u >> 2) * p.Bp + b) * 4 + (u & 3);
      for (int k = 0; k < kStepBuffers - 1; ++k) x[k * p.bufsz + slot] = kSentinel;
      // step 0 reads buffer (0 - 1) mod 4 = 3
      p.xbase[d][(size_t)(kStepBuffers - 1) * p.bufsz + slot] = p.h0[d] ? p.h0[d][gtid] : 0.f;
    } else {
      const size_t slot = ((size_t)u * p.Bp + b) * 4;
      for (int k = 0; k < kStepBuffers; ++k)
        for (int g = 0; g < 4; ++g) x[k * p.bufsz + slot + g] = kSentinel;
    }
  }
}

// ---- host side ----------------------------------------------------------------
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Plan {
  bool ok;
  int MT, NT, U, UG, Bp;
  int Gf, Hp;
  int PG, Gb, Hq;
  size_t ldsF, ldsB;
};

Plan make_plan(const RecShape& s, int num_cus, size_t max_lds) {
  Plan pl{};
  pl.ok = false;
  if (s.operand_dtype != 0) return pl;
  if (s.B < 1 || s.B > 64 || s.H < 1) return pl;
  pl.MT = s.B <= 16 ? 1 : (s.B <= 32 ? 2 : 4);
  pl.Bp = pl.MT * 16;
  const int per_dir = num_cus / s.ndir;
  for (int NT = 1; NT <= 2; ++NT) {
    const int U = 4 * NT, UG = 16 * NT;
    const int Gf = (s.H + U - 1) / U;
    const int PG = (s.H + UG - 1) / UG;
    const int Gb = 4 * PG;
    if (Gf > per_dir || Gb > per_dir) continue;
    const int Hp = (int)align_up((size_t)s.H, 64);
    const int Hq = (int)align_up((size_t)PG * U, 32);
    const size_t red = (size_t)4 * pl.MT * NT * 256;
    const size_t lf = ((size_t)Hp * 16 * NT + red + (size_t)(2 * 4 + 2 * 6) * pl.MT * 16 * U) * sizeof(float);
    const size_t lb = ((size_t)4 * Hq * UG + red + (size_t)(2 * 7 + 2 * 4) * pl.MT * 16 * U) * sizeof(float);
    if (lf > max_lds || lb > max_lds) continue;
    // One workgroup per CU: request more than half of the CU's LDS so that the dispatcher cannot
    // stack two of these workgroups on one CU (they would share its matrix cores and every other
    // workgroup would wait for them each step).
    const size_t exclusive = max_lds / 2 + 1024;
    const size_t lf_req = lf > exclusive ? lf : exclusive, lb_req = lb > exclusive ? lb : exclusive;
    pl.ok = true; pl.NT = NT; pl.U = U; pl.UG = UG;
    pl.Gf = Gf; pl.Hp = Hp;
    pl.PG = PG; pl.Gb = Gb; pl.Hq = Hq;
    pl.ldsF = lf_req; pl.ldsB = lb_req;
    return pl;
  }
  return pl;
}

// Launches a kernel whose workgroups wait on each other.  All of them must be resident at
// once: the grid may not exceed what the device can hold of this kernel (checked here).
// A plain launch is used; other work on the device can delay residency but not prevent it,
// and the kernels' own waits are bounded.
template <typename K>
hipError_t resident_launch(K kernel, int grid, int block, size_t lds, int num_cus, hipStream_t stream, void* params,
                           int* resident_err) {
  hipError_t e = hipSuccess;
  const void* fn = reinterpret_cast<const void*>(kernel);
  if (lds > 48 * 1024) {
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  int per_cu = 0;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, block, lds);
  if (e != hipSuccess) return e;
  if ((long long)per_cu * num_cus < grid) { *resident_err = 1; return hipErrorCooperativeLaunchTooLarge; }
  void* args[] = {params};
  return hipLaunchKernel(fn, dim3((unsigned)grid), dim3((unsigned)block), args, lds, stream);
}

}  // namespace

bool persistent_supported(const RecShape& s, int num_cus, size_t max_lds) {
  return make_plan(s, num_cus, max_lds).ok;
}

// Upper bound (independent of the device) of the per-direction scratch, in bytes:
// [exchange arrays][partial tiles].
size_t persistent_scratch_bytes_per_dir(const RecShape& s) {
  const size_t Bp = s.B <= 16 ? 16 : (s.B <= 32 ? 32 : 64);
  const size_t Hp = align_up((size_t)s.H, 64);
  const size_t Hq = align_up((size_t)s.H / 4 + 8, 32);
  const size_t exch = kStepBuffers * (Hp > 16 * Hq ? Hp : 16 * Hq) * Bp * sizeof(float);
  const size_t part = 2 * 4 * Bp * ((size_t)s.H + 32) * sizeof(unsigned long long);
  return align_up(exch, 256) + align_up(part, 256);
}

hipError_t persistent_forward(hipStream_t stream, const RecShape& s, const RecFwdDir* dirs, const int32_t* seq_lens,
                              char* const* scratch, unsigned* err, int* resident_err) {
  DeviceInfo di;
  hipError_t e = device_info(&di);
  if (e != hipSuccess) return e;
  const Plan pl = make_plan(s, di.num_cus, di.max_lds);
  if (!pl.ok) { *resident_err = 1; return hipErrorInvalidValue; }
  const size_t bufsz = (size_t)pl.Hp * pl.Bp;
  PrepParams pp{};
  PFwdParams kp{};
  for (int d = 0; d < s.ndir; ++d) {
    float* hx = reinterpret_cast<float*>(scratch[d]);
    pp.zero_words[d] = reinterpret_cast<unsigned*>(hx);
    pp.nzero[d] = (size_t)kStepBuffers * bufsz;
    pp.xbase[d] = hx;
    pp.h0[d] = dirs[d].h0;
    PFwdDir& k = kp.d[d];
    k.zg = dirs[d].zg; k.R = dirs[d].R; k.h0 = dirs[d].h0; k.c0 = dirs[d].c0;
    k.y = dirs[d].y; k.c = dirs[d].c; k.hT = dirs[d].hT; k.cT = dirs[d].cT;
    k.hx = hx; k.direction = dirs[d].direction;
  }
  pp.ndir = s.ndir; pp.B = s.B; pp.H = s.H; pp.Bp = pl.Bp; pp.backward = 0; pp.bufsz = bufsz;
  kp.seq_lens = seq_lens; kp.err = err;
  kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy; kp.Gf = pl.Gf; kp.Hp = pl.Hp;
  hipLaunchKernelGGL(prep_kernel, dim3(64), dim3(256), 0, stream, pp);
  {
    const size_t bh = (size_t)s.B * s.H;
    hipLaunchKernelGGL(seed_kernel, dim3((unsigned)((bh + 255) / 256)), dim3(256), 0, stream, pp);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int grid = pl.Gf * s.ndir;
#define RLSTM_FWD_CASE(MT_, NT_)                                                                      \
  if (pl.MT == MT_ && pl.NT == NT_)                                                                   \
    return resident_launch(lstm_fwd_persistent_kernel<MT_, NT_>, grid, kBlockThreads, pl.ldsF, di.num_cus, stream, &kp, resident_err);
  RLSTM_FWD_CASE(1, 1) RLSTM_FWD_CASE(2, 1) RLSTM_FWD_CASE(4, 1)
  RLSTM_FWD_CASE(1, 2) RLSTM_FWD_CASE(2, 2) RLSTM_FWD_CASE(4, 2)
#undef RLSTM_FWD_CASE
  return hipErrorInvalidValue;
}

hipError_t persistent_backward(hipStream_t stream, const RecShape& s, const RecBwdDir* dirs, const int32_t* seq_lens,
                               char* const* scratch, unsigned* err, int* resident_err) {
  DeviceInfo di;
  hipError_t e = device_info(&di);
  if (e != hipSuccess) return e;
  const Plan pl = make_plan(s, di.num_cus, di.max_lds);
  if (!pl.ok) { *resident_err = 1; return hipErrorInvalidValue; }
  const size_t bufsz = (size_t)16 * pl.Hq * pl.Bp;
  const size_t exch_floats = (size_t)kStepBuffers * bufsz;
  const size_t part_words = (size_t)2 * pl.PG * 4 * pl.Bp * pl.UG;
  PrepParams pp{};
  PBwdParams kp{};
  for (int d = 0; d < s.ndir; ++d) {
    float* dzx = reinterpret_cast<float*>(scratch[d]);
    unsigned long long* part = reinterpret_cast<unsigned long long*>(dzx + align_up(exch_floats, 64));
    pp.zero_words[d] = reinterpret_cast<unsigned*>(dzx);
    pp.nzero[d] = align_up(exch_floats, 64) + 2 * part_words;
    pp.xbase[d] = dzx; pp.h0[d] = nullptr;
    PBwdDir& k = kp.d[d];
    k.zg = dirs[d].zg; k.R = dirs[d].R; k.c = dirs[d].c; k.c0 = dirs[d].c0; k.dy = dirs[d].dy;
    k.dhT = dirs[d].dhT; k.dcT = dirs[d].dcT; k.dh0 = dirs[d].dh0; k.dc0 = dirs[d].dc0; k.db = dirs[d].db;
    k.dzx = dzx; k.part = part; k.direction = dirs[d].direction;
  }
  pp.ndir = s.ndir; pp.B = s.B; pp.H = s.H; pp.Bp = pl.Bp; pp.backward = 1; pp.bufsz = bufsz;
  kp.seq_lens = seq_lens; kp.err = err;
  kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy; kp.PG = pl.PG; kp.Hq = pl.Hq;
  hipLaunchKernelGGL(prep_kernel, dim3(128), dim3(256), 0, stream, pp);
  {
    const size_t bh = (size_t)s.B * s.H;
    hipLaunchKernelGGL(seed_kernel, dim3((unsigned)((bh + 255) / 256)), dim3(256), 0, stream, pp);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int grid = pl.Gb * s.ndir;
#define RLSTM_BWD_CASE(MT_, NT_)                                                                      \
  if (pl.MT == MT_ && pl.NT == NT_)                                                                   \
    return resident_launch(lstm_bwd_persistent_kernel<MT_, NT_>, grid, kBlockThreads, pl.ldsB, di.num_cus, stream, &kp, resident_err);
  RLSTM_BWD_CASE(1, 1) RLSTM_BWD_CASE(2, 1) RLSTM_BWD_CASE(4, 1)
  RLSTM_BWD_CASE(1, 2) RLSTM_BWD_CASE(2, 2) RLSTM_BWD_CASE(4, 2)
#undef RLSTM_BWD_CASE
  return hipErrorInvalidValue;
}

}  // namespace rlstm
