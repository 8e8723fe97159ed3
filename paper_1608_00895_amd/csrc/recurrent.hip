// The recurrent part of the LSTM layer (Sec. 4.2 of the RETURNN paper): the
// time loop h_{t-1} R + gating forwards, and the pass back through time.
//
// Persistent engine.  One cooperative launch runs all T steps of up to two
// independent directions.  The units of a direction are dealt out to G
// workgroups, U units each (U = 4 or 8): a workgroup owns the i, f, o, g
// columns of its units, keeps that slice of R (forward) or of R^T (backward)
// in LDS for the whole kernel, keeps c, h, dc, dh of its units in registers,
// and does its share of the per-step product on the matrix cores
// (v_mfma_f32_16x16x4_f32, K split over the 4 wavefronts, partial tiles summed
// through LDS in a fixed order).  Between steps the full h_t (forward) or
// d loss / d a_t (backward) is exchanged through a double-buffered, k-major
// [K][batch] array in global memory, published and consumed around a
// device-wide barrier (agent-scope release / acquire on one counter per
// direction).  Sigmoid / tanh, the cell update, the validity mask (Sec. 5) and
// the stores of gates, y and c are fused behind the product of the same step.
//
// Stepwise engine.  The same mathematics as one plain launch per time step
// (one thread per (sequence, unit)); it accepts any shape and is the on-device
// cross-check of the persistent engine.
#include "rlstm_internal.h"

namespace rlstm {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ float sigmoidf_(float u) { return 1.0f / (1.0f + expf(-u)); }

constexpr int KCH = 8;                 // k-steps (of 4) per software-pipelined chunk of the per-step product
constexpr int KALIGN = 4 * 4 * KCH;    // padded K: 4 wavefronts x whole chunks
constexpr unsigned long long kBarrierTimeoutTicks = 400000000ull;   // 4 s of the 100 MHz wall clock

// ---------------------------------------------------------------------------
// device-wide barrier of the G workgroups of one direction
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool group_barrier(unsigned* ctr, unsigned target, unsigned* flag, int* lds_ok) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int ok = 1;
    unsigned spins = 0;
    unsigned long long t0 = 0;
    while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      __builtin_amdgcn_s_sleep(1);
      if ((++spins & 255u) == 0) {
        const unsigned long long now = wall_clock64();
        if (t0 == 0) t0 = now;
        else if (now - t0 > kBarrierTimeoutTicks) { ok = 0; break; }
        if (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) { ok = 0; break; }
      }
    }
    if (!ok) __hip_atomic_store(flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *lds_ok = ok;
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  return *lds_ok != 0;
}

// ---------------------------------------------------------------------------
// persistent forward
// ---------------------------------------------------------------------------
struct PFwdDir {
  float* zg; const float* R; const float* h0; const float* c0;
  float* y; float* c; float* hT; float* cT;
  float* hx;            // 2 x [Hp][Bp]
  unsigned* bar;
  int direction;
};
struct PFwdParams {
  PFwdDir d[2];
  const int32_t* seq_lens;
  unsigned* flag;
  int T, B, H, ldy, G, Bp, Hp;
};

// MT: 16-row batch tiles (B <= 16*MT).  NT: 16-column tiles; U = 4*NT units per workgroup.
template <int MT, int NT>
__global__ __launch_bounds__(256) void lstm_fwd_persistent_kernel(PFwdParams p) {
  constexpr int U = 4 * NT, NC = 16 * NT;
  constexpr int EPT = (MT * 16 * U + 255) / 256;
  extern __shared__ __align__(16) float lds[];
  const int dir = blockIdx.x / p.G, wg = blockIdx.x % p.G;
  const PFwdDir& D = p.d[dir];
  const int T = p.T, B = p.B, H = p.H, Bp = p.Bp, Hp = p.Hp;
  const int u0 = wg * U;
  float* Rs = lds;                               // [Hp][NC]
  float* Red = lds + (size_t)Hp * NC;            // [4][MT][NT][64][4]
  int* lds_ok = reinterpret_cast<int*>(Red + 4 * MT * NT * 256);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lq = lane >> 4;

  // resident slice of R: slice column g*U + uu is column g*H + u0 + uu of R
  for (int idx = tid; idx < Hp * NC; idx += 256) {
    const int k = idx / NC, col = idx % NC;
    const int g = col / U, u = u0 + col % U;
    Rs[idx] = (k < H && u < H) ? D.R[(size_t)k * 4 * H + g * H + u] : 0.f;
  }

  // carried state of the (sequence, unit) pairs this thread owns
  float hreg[EPT], creg[EPT];
  int eb[EPT], eu[EPT], elen[EPT];
  bool ev[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int j = tid + e * 256;
    eb[e] = j / U; eu[e] = u0 + j % U;
    ev[e] = (j < MT * 16 * U) && eb[e] < B && eu[e] < H;
    hreg[e] = 0.f; creg[e] = 0.f; elen[e] = 0;
    if (ev[e]) {
      if (D.h0) hreg[e] = D.h0[(size_t)eb[e] * H + eu[e]];
      if (D.c0) creg[e] = D.c0[(size_t)eb[e] * H + eu[e]];
      elen[e] = min(max(p.seq_lens[eb[e]], 0), T);
    }
  }
  __syncthreads();

  const int KW = Hp / 4;                 // k range of one wavefront (multiple of 4)
  const int kbase = wave * KW;
  const size_t hxsz = (size_t)Hp * Bp;

  for (int s = 0; s < T; ++s) {
    const int t = D.direction > 0 ? s : T - 1 - s;
    const float* hprev = D.hx + (size_t)((s + 1) & 1) * hxsz;
    float* hcur = D.hx + (size_t)(s & 1) * hxsz;

    // non-recurrent part of this frame (computed beforehand for all frames)
    float za[EPT][4];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
        za[e][g] = ev[e] ? D.zg[((size_t)t * B + eb[e]) * 4 * H + g * H + eu[e]] : 0.f;
    }

    // recurrent part: this wavefront's K range of h_prev [B x H] * R[:, slice]
    floatx4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
    // KW is a multiple of 4*KCH: chunks of KCH k-steps, all loads of a chunk issued before its MFMAs
    for (int kc = 0; kc < KW; kc += 4 * KCH) {
      float bf[KCH][NT], af[KCH][MT];
#pragma unroll
      for (int q = 0; q < KCH; ++q) {
        const int k = kbase + kc + 4 * q + lq;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) af[q][mt] = hprev[(size_t)k * Bp + mt * 16 + l16];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bf[q][nt] = Rs[k * NC + nt * 16 + l16];
      }
#pragma unroll
      for (int q = 0; q < KCH; ++q)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[q][mt], bf[q][nt], acc[mt][nt], 0, 0, 0);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        *reinterpret_cast<floatx4*>(Red + (((wave * MT + mt) * NT + nt) * 64 + lane) * 4) = acc[mt][nt];
    __syncthreads();

    // gating, cell update, mask, stores
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if (!ev[e]) continue;
      const int b = eb[e], u = eu[e], uu = u - u0;
      const int mt = b >> 4, r = b & 15;
      float a[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = g * U + uu;
        const int nt = col >> 4, n = col & 15;
        const int src = ((r >> 2) * 16 + n) * 4 + (r & 3);    // accumulator (row r, col n) of a 16x16 tile
        float sum = za[e][g];
#pragma unroll
        for (int w = 0; w < 4; ++w) sum += Red[((w * MT + mt) * NT + nt) * 256 + src];
        a[g] = sum;
      }
      const float gi = sigmoidf_(a[0]), gf = sigmoidf_(a[1]), go = sigmoidf_(a[2]), gg = tanhf(a[3]);
      const float cn = gf * creg[e] + gi * gg;
      const float hn = go * tanhf(cn);
      const bool valid = t < elen[e];
      if (valid) { creg[e] = cn; hreg[e] = hn; }
      const size_t row = (size_t)t * B + b;
      float* zrow = D.zg + row * 4 * H + u;
      zrow[0] = gi; zrow[H] = gf; zrow[2 * H] = go; zrow[3 * H] = gg;
      D.y[row * p.ldy + u] = valid ? hn : 0.f;
      D.c[row * H + u] = creg[e];
      hcur[(size_t)u * Bp + b] = hreg[e];
    }

    if (!group_barrier(D.bar, (unsigned)p.G * (unsigned)(s + 1), p.flag, lds_ok)) return;
  }

#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    if (!ev[e]) continue;
    if (D.hT) D.hT[(size_t)eb[e] * H + eu[e]] = hreg[e];
    if (D.cT) D.cT[(size_t)eb[e] * H + eu[e]] = creg[e];
  }
}

// zero the exchange buffers and the barrier counters; seed buffer 1 with h0 (k-major)
struct PrepFwdParams {
  float* hx[2]; const float* h0[2]; unsigned* bar[2];
  int ndir, B, H, Bp, Hp;
};
__global__ __launch_bounds__(256) void prep_fwd_kernel(PrepFwdParams p) {
  const size_t hxsz = (size_t)p.Hp * p.Bp;
  for (int d = 0; d < p.ndir; ++d) {
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < 2 * hxsz; idx += (size_t)gridDim.x * 256) {
      float v = 0.f;
      if (idx >= hxsz && p.h0[d]) {
        const size_t r = idx - hxsz;
        const int k = (int)(r / p.Bp), b = (int)(r % p.Bp);
        if (k < p.H && b < p.B) v = p.h0[d][(size_t)b * p.H + k];
      }
      p.hx[d][idx] = v;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) *p.bar[d] = 0u;
  }
}

// ---------------------------------------------------------------------------
// persistent backward (back-propagation through time)
// ---------------------------------------------------------------------------
struct PBwdDir {
  float* zg; const float* R; const float* c; const float* c0; const float* dy;
  const float* dhT; const float* dcT; float* dh0; float* dc0; float* db;
  float* dzx;           // 2 x [Kp][Bp]
  unsigned* bar;
  int direction;
};
struct PBwdParams {
  PBwdDir d[2];
  const int32_t* seq_lens;
  unsigned* flag;
  int T, B, H, ldy, G, Bp, Kp;
};

template <int MT, int U>
__global__ __launch_bounds__(256) void lstm_bwd_persistent_kernel(PBwdParams p) {
  constexpr int EPT = (MT * 16 * U + 255) / 256;
  extern __shared__ __align__(16) float lds[];
  const int dir = blockIdx.x / p.G, wg = blockIdx.x % p.G;
  const PBwdDir& D = p.d[dir];
  const int T = p.T, B = p.B, H = p.H, Bp = p.Bp, Kp = p.Kp;
  const int u0 = wg * U;
  float* RTs = lds;                              // [Kp][U]: RTs[kx][n] = R[u0+n][column of kx]
  float* Red = lds + (size_t)Kp * U;             // [4][MT][64][4]
  int* lds_ok = reinterpret_cast<int*>(Red + 4 * MT * 256);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lq = lane >> 4;

  // exchange index kx = wgp*4U + g*U + uu  <->  column g*H + wgp*U + uu of the 4H gate columns
  for (int idx = tid; idx < Kp * U; idx += 256) {
    const int kx = idx / U, n = idx % U;
    const int wgp = kx / (4 * U), rem = kx % (4 * U);
    const int g = rem / U, uc = wgp * U + rem % U;
    const int un = u0 + n;
    RTs[idx] = (uc < H && un < H) ? D.R[(size_t)un * 4 * H + g * H + uc] : 0.f;
  }

  float Dh[EPT], Dc[EPT], dbacc[EPT][4];
  int eb[EPT], eu[EPT], elen[EPT];
  bool ev[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int j = tid + e * 256;
    eb[e] = j / U; eu[e] = u0 + j % U;
    ev[e] = (j < MT * 16 * U) && eb[e] < B && eu[e] < H;
    Dh[e] = 0.f; Dc[e] = 0.f; elen[e] = 0;
#pragma unroll
    for (int g = 0; g < 4; ++g) dbacc[e][g] = 0.f;
    if (ev[e]) {
      if (D.dhT) Dh[e] = D.dhT[(size_t)eb[e] * H + eu[e]];
      if (D.dcT) Dc[e] = D.dcT[(size_t)eb[e] * H + eu[e]];
      elen[e] = min(max(p.seq_lens[eb[e]], 0), T);
    }
  }
  __syncthreads();

  const int KW = Kp / 4;
  const int kbase = wave * KW;
  const size_t xsz = (size_t)Kp * Bp;

  for (int s = 0; s < T; ++s) {
    // frames are visited in the reverse of the forward processing order
    const int t = D.direction > 0 ? T - 1 - s : s;
    const int tprev = D.direction > 0 ? t - 1 : t + 1;     // frame processed before t in the forward pass
    float* dzcur = D.dzx + (size_t)(s & 1) * xsz;
    bool valid[EPT];

#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      valid[e] = false;
      if (!ev[e]) continue;
      const int b = eb[e], u = eu[e], uu = u - u0;
      const size_t row = (size_t)t * B + b;
      float* zrow = D.zg + row * 4 * H + u;
      const float gi = zrow[0], gf = zrow[H], go = zrow[2 * H], gg = zrow[3 * H];
      const float ct = D.c[row * H + u];
      float cp;
      if (tprev >= 0 && tprev < T) cp = D.c[((size_t)tprev * B + b) * H + u];
      else cp = D.c0 ? D.c0[(size_t)b * H + u] : 0.f;
      const float dyv = D.dy[row * p.ldy + u];
      const bool m = t < elen[e];
      valid[e] = m;
      float dz[4] = {0.f, 0.f, 0.f, 0.f};
      if (m) {
        const float tc = tanhf(ct);
        const float dh = dyv + Dh[e];
        const float d_o = dh * tc;
        const float dc = Dc[e] + dh * go * (1.0f - tc * tc);
        dz[0] = dc * gg * gi * (1.0f - gi);
        dz[1] = dc * cp * gf * (1.0f - gf);
        dz[2] = d_o * go * (1.0f - go);
        dz[3] = dc * gi * (1.0f - gg * gg);
        Dc[e] = dc * gf;
      }
      zrow[0] = dz[0]; zrow[H] = dz[1]; zrow[2 * H] = dz[2]; zrow[3 * H] = dz[3];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        dzcur[(size_t)(wg * 4 * U + g * U + uu) * Bp + b] = dz[g];
        dbacc[e][g] += dz[g];
      }
    }

    if (!group_barrier(D.bar, (unsigned)p.G * (unsigned)(s + 1), p.flag, lds_ok)) return;

    // Dh <- dz_t R^T (+ carried Dh where the frame was invalid)
    floatx4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int kc = 0; kc < KW; kc += 4 * KCH) {
      float bf[KCH], af[KCH][MT];
#pragma unroll
      for (int q = 0; q < KCH; ++q) {
        const int k = kbase + kc + 4 * q + lq;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) af[q][mt] = dzcur[(size_t)k * Bp + mt * 16 + l16];
        bf[q] = (l16 < U) ? RTs[k * U + l16] : 0.f;
      }
#pragma unroll
      for (int q = 0; q < KCH; ++q)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[q][mt], bf[q], acc[mt], 0, 0, 0);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      *reinterpret_cast<floatx4*>(Red + ((wave * MT + mt) * 64 + lane) * 4) = acc[mt];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if (!ev[e]) continue;
      const int b = eb[e], uu = eu[e] - u0;
      const int mt = b >> 4, r = b & 15;
      const int src = ((r >> 2) * 16 + uu) * 4 + (r & 3);
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) sum += Red[(w * MT + mt) * 256 + src];
      Dh[e] = valid[e] ? sum : sum + Dh[e];
    }
    // Red is rewritten only after the next step's barrier (which synchronises the workgroup)
  }

  // outputs: gradient w.r.t. the initial state, and the bias gradient of this slice
  __syncthreads();
  float* stage = Red;                            // [Bp][4U]
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int j = tid + e * 256;
    if (j < MT * 16 * U) {
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

struct PrepBwdParams {
  float* dzx[2]; unsigned* bar[2];
  int ndir; size_t floats;
};
__global__ __launch_bounds__(256) void prep_bwd_kernel(PrepBwdParams p) {
  for (int d = 0; d < p.ndir; ++d) {
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < p.floats; idx += (size_t)gridDim.x * 256)
      p.dzx[d][idx] = 0.f;
    if (blockIdx.x == 0 && threadIdx.x == 0) *p.bar[d] = 0u;
  }
}

// ---------------------------------------------------------------------------
// stepwise engine: one launch per time step, one thread per (sequence, unit)
// ---------------------------------------------------------------------------
struct SFwdDir {
  float* zg; const float* R; const float* c0; float* y; float* c; float* hT; float* cT;
  float* hbuf;          // 2 x [B,H] carried h, double-buffered
  int direction;
};
struct SFwdParams { SFwdDir d[2]; const int32_t* seq_lens; int T, B, H, ldy, s; };

__global__ __launch_bounds__(256) void step_fwd_kernel(SFwdParams p) {
  const SFwdDir& D = p.d[blockIdx.y];
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int B = p.B, H = p.H, T = p.T;
  if (j >= B * H) return;
  const int b = j / H, u = j % H;
  const int s = p.s;
  const int t = D.direction > 0 ? s : T - 1 - s;
  const int tprev = D.direction > 0 ? t - 1 : t + 1;
  const float* hprev = D.hbuf + (size_t)((s + 1) & 1) * B * H;
  float* hcur = D.hbuf + (size_t)(s & 1) * B * H;
  const size_t row = (size_t)t * B + b;
  float* zrow = D.zg + row * 4 * H + u;
  float a0 = zrow[0], a1 = zrow[H], a2 = zrow[2 * H], a3 = zrow[3 * H];
  for (int k = 0; k < H; ++k) {
    const float hv = hprev[(size_t)b * H + k];
    const float* rr = D.R + (size_t)k * 4 * H + u;
    a0 = fmaf(hv, rr[0], a0); a1 = fmaf(hv, rr[H], a1); a2 = fmaf(hv, rr[2 * H], a2); a3 = fmaf(hv, rr[3 * H], a3);
  }
  float cprev;
  if (tprev >= 0 && tprev < T) cprev = D.c[((size_t)tprev * B + b) * H + u];
  else cprev = D.c0 ? D.c0[(size_t)b * H + u] : 0.f;
  const float gi = sigmoidf_(a0), gf = sigmoidf_(a1), go = sigmoidf_(a2), gg = tanhf(a3);
  const float cn = gf * cprev + gi * gg;
  const float hn = go * tanhf(cn);
  const int len = min(max(p.seq_lens[b], 0), T);
  const bool valid = t < len;
  const float cs = valid ? cn : cprev;
  const float hs = valid ? hn : hprev[(size_t)b * H + u];
  zrow[0] = gi; zrow[H] = gf; zrow[2 * H] = go; zrow[3 * H] = gg;
  D.y[row * p.ldy + u] = valid ? hn : 0.f;
  D.c[row * H + u] = cs;
  hcur[(size_t)b * H + u] = hs;
  if (s == T - 1) {
    if (D.hT) D.hT[(size_t)b * H + u] = hs;
    if (D.cT) D.cT[(size_t)b * H + u] = cs;
  }
}

struct SInitParams { float* dst[2]; const float* src[2]; int ndir; size_t n; size_t off; };
// dst[d][off + i] = src[d] ? src[d][i] : 0
__global__ __launch_bounds__(256) void init_state_kernel(SInitParams p) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= p.n) return;
  for (int d = 0; d < p.ndir; ++d) p.dst[d][p.off + i] = p.src[d] ? p.src[d][i] : 0.f;
}

struct SBwdDir {
  float* zg; const float* R; const float* c; const float* c0; const float* dy;
  float* dh0; float* dc0;
  float* dhbuf;         // 2 x [B,H] carried Dh, double-buffered
  float* dcbuf;         // [B,H] carried Dc
  int direction;
};
struct SBwdParams { SBwdDir d[2]; const int32_t* seq_lens; int T, B, H, ldy, s; };

// gate derivatives of step s: reads Dh of buffer (s+1)&1, writes dz in place and updates Dc
__global__ __launch_bounds__(256) void step_bwd_gates_kernel(SBwdParams p) {
  const SBwdDir& D = p.d[blockIdx.y];
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int B = p.B, H = p.H, T = p.T;
  if (j >= B * H) return;
  const int b = j / H, u = j % H;
  const int s = p.s;
  const int t = D.direction > 0 ? T - 1 - s : s;
  const int tprev = D.direction > 0 ? t - 1 : t + 1;
  const float Dh = D.dhbuf[(size_t)((s + 1) & 1) * B * H + j];
  const size_t row = (size_t)t * B + b;
  float* zrow = D.zg + row * 4 * H + u;
  const float gi = zrow[0], gf = zrow[H], go = zrow[2 * H], gg = zrow[3 * H];
  const float ct = D.c[row * H + u];
  float cp;
  if (tprev >= 0 && tprev < T) cp = D.c[((size_t)tprev * B + b) * H + u];
  else cp = D.c0 ? D.c0[(size_t)b * H + u] : 0.f;
  const int len = min(max(p.seq_lens[b], 0), T);
  float dz0 = 0.f, dz1 = 0.f, dz2 = 0.f, dz3 = 0.f;
  if (t < len) {
    const float tc = tanhf(ct);
    const float dh = D.dy[row * p.ldy + u] + Dh;
    const float d_o = dh * tc;
    const float dc = D.dcbuf[j] + dh * go * (1.0f - tc * tc);
    dz0 = dc * gg * gi * (1.0f - gi);
    dz1 = dc * cp * gf * (1.0f - gf);
    dz2 = d_o * go * (1.0f - go);
    dz3 = dc * gi * (1.0f - gg * gg);
    D.dcbuf[j] = dc * gf;
  }
  zrow[0] = dz0; zrow[H] = dz1; zrow[2 * H] = dz2; zrow[3 * H] = dz3;
  if (s == T - 1 && D.dc0) D.dc0[j] = D.dcbuf[j];
}

// Dh of buffer s&1 = dz_t R^T (+ Dh of buffer (s+1)&1 where the frame was invalid)
__global__ __launch_bounds__(256) void step_bwd_dh_kernel(SBwdParams p) {
  const SBwdDir& D = p.d[blockIdx.y];
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int B = p.B, H = p.H, T = p.T;
  if (j >= B * H) return;
  const int b = j / H, u = j % H;
  const int s = p.s;
  const int t = D.direction > 0 ? T - 1 - s : s;
  const float* dz = D.zg + ((size_t)t * B + b) * 4 * H;
  const float* rr = D.R + (size_t)u * 4 * H;
  float sum = 0.f;
  for (int k = 0; k < 4 * H; ++k) sum = fmaf(dz[k], rr[k], sum);
  const int len = min(max(p.seq_lens[b], 0), T);
  if (!(t < len)) sum += D.dhbuf[(size_t)((s + 1) & 1) * B * H + j];
  D.dhbuf[(size_t)(s & 1) * B * H + j] = sum;
  if (s == T - 1 && D.dh0) D.dh0[j] = sum;
}

__global__ __launch_bounds__(256) void column_sum_kernel(const float* __restrict__ a, size_t rows, int cols, int lda,
                                                          float* __restrict__ out) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= cols) return;
  float s = 0.f;
  for (size_t r = 0; r < rows; ++r) s += a[r * lda + n];
  out[n] = s;
}

// dR[k][n] += sum_b h0[b][k] * dz[tfirst(b)][b][n], tfirst = first processed valid frame
__global__ __launch_bounds__(256) void add_h0_outer_kernel(int T, int B, int H, int direction, const float* __restrict__ h0,
                                                            const float* __restrict__ dz, const int32_t* __restrict__ seq_lens,
                                                            float* __restrict__ dR) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)H * 4 * H) return;
  const int k = (int)(idx / (4 * H)), n = (int)(idx % (4 * H));
  float s = 0.f;
  for (int b = 0; b < B; ++b) {
    const int len = min(max(seq_lens[b], 0), T);
    if (len == 0) continue;
    const int tf = direction > 0 ? 0 : len - 1;
    s = fmaf(h0[(size_t)b * H + k], dz[((size_t)tf * B + b) * 4 * H + n], s);
  }
  dR[idx] += s;
}

__global__ void clear_flag_kernel(unsigned* flag) { *flag = 0u; }

// ---- host-side layout of the recurrent scratch ------------------------------
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct PersistentPlan {
  bool ok;
  int MT, U, G, Bp, Hp, Kp;
  size_t lds_fwd, lds_bwd;
};

PersistentPlan plan_persistent(const RecShape& s, int num_cus, size_t max_lds) {
  PersistentPlan pl{};
  pl.ok = false;
  if (s.operand_dtype != 0) return pl;
  if (s.B < 1 || s.B > 64 || s.H < 1) return pl;
  pl.MT = s.B <= 16 ? 1 : (s.B <= 32 ? 2 : 4);
  pl.Bp = pl.MT * 16;
  const int per_dir = num_cus / s.ndir;
  for (int U = 4; U <= 8; U += 4) {
    const int G = (s.H + U - 1) / U;
    if (G > per_dir) continue;
    const int NT = U / 4;
    const int Hp = (int)align_up((size_t)s.H, KALIGN);
    const int Kp = (int)align_up((size_t)G * 4 * U, KALIGN);
    const size_t lf = ((size_t)Hp * 16 * NT + (size_t)4 * pl.MT * NT * 256) * sizeof(float) + 16;
    const size_t lb = ((size_t)Kp * U + (size_t)4 * pl.MT * 256) * sizeof(float) + 16;
    if (lf > max_lds || lb > max_lds) continue;
    pl.ok = true; pl.U = U; pl.G = G; pl.Hp = Hp; pl.Kp = Kp; pl.lds_fwd = lf; pl.lds_bwd = lb;
    return pl;
  }
  return pl;
}

// scratch: [bar0 | bar1] (256 B) then per direction the larger of the two engines' needs
struct RecScratch {
  unsigned* bar[2];
  float* buf[2];
  size_t per_dir_floats;
};
size_t rec_per_dir_floats(const RecShape& s) {
  // persistent: max(2*Hp*Bp, 2*Kp*Bp) with the most generous padding; stepwise: 2*B*H (h or Dh) + B*H (Dc)
  const size_t Bp = s.B <= 16 ? 16 : (s.B <= 32 ? 32 : (s.B <= 64 ? 64 : align_up((size_t)s.B, 16)));
  const size_t Hp = align_up((size_t)s.H, KALIGN);
  const size_t Kp = align_up(4 * (align_up((size_t)s.H, 8) + 8), KALIGN);
  size_t a = 2 * Kp * Bp;
  size_t b = 2 * Hp * Bp;
  size_t c = 3 * (size_t)s.B * s.H;
  size_t m = a > b ? a : b;
  m = m > c ? m : c;
  return align_up(m, 64);
}
RecScratch carve(const RecShape& s, void* ws) {
  RecScratch r;
  char* base = static_cast<char*>(ws);
  r.bar[0] = reinterpret_cast<unsigned*>(base);
  r.bar[1] = reinterpret_cast<unsigned*>(base + 128);
  r.per_dir_floats = rec_per_dir_floats(s);
  r.buf[0] = reinterpret_cast<float*>(base + 256);
  r.buf[1] = r.buf[0] + r.per_dir_floats;
  return r;
}

template <typename K>
hipError_t coop_launch(K kernel, int grid, size_t lds, hipStream_t stream, void* params, int* resident_err) {
  hipError_t e = hipSuccess;
  if (lds > 48 * 1024) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  void* args[] = {params};
  e = hipLaunchCooperativeKernel(reinterpret_cast<const void*>(kernel), dim3((unsigned)grid), dim3(256), args,
                                 (unsigned)lds, stream);
  if (e == hipErrorCooperativeLaunchTooLarge) { *resident_err = 1; (void)hipGetLastError(); }
  return e;
}

}  // namespace

size_t rec_workspace_bytes(const RecShape& s) {
  return 256 + 2 * rec_per_dir_floats(s) * sizeof(float);
}

bool rec_persistent_supported(const RecShape& s, int num_cus, size_t max_lds) {
  return plan_persistent(s, num_cus, max_lds).ok;
}

hipError_t device_info(DeviceInfo* out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  int cus = 0, lds = 0;
  e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
  if (e != hipSuccess) return e;
  out->num_cus = cus;
  out->max_lds = (size_t)lds;
  return hipSuccess;
}

hipError_t clear_flag(hipStream_t stream, unsigned* flag) {
  hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, stream, flag);
  return hipGetLastError();
}

hipError_t column_sum(hipStream_t stream, const float* a, size_t rows, int cols, int lda, float* out) {
  hipLaunchKernelGGL(column_sum_kernel, dim3((unsigned)((cols + 255) / 256)), dim3(256), 0, stream, a, rows, cols, lda, out);
  return hipGetLastError();
}

hipError_t add_h0_outer(hipStream_t stream, int T, int B, int H, int direction, const float* h0,
                        const float* dz, const int32_t* seq_lens, float* dR) {
  const size_t total = (size_t)H * 4 * H;
  hipLaunchKernelGGL(add_h0_outer_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                     T, B, H, direction, h0, dz, seq_lens, dR);
  return hipGetLastError();
}

hipError_t rec_forward(hipStream_t stream, const RecShape& s, const RecFwdDir* dirs, const int32_t* seq_lens,
                       void* ws, unsigned* flag, bool persistent, int* resident_err) {
  RecScratch sc = carve(s, ws);
  if (persistent) {
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    PersistentPlan pl = plan_persistent(s, di.num_cus, di.max_lds);
    if (!pl.ok) { *resident_err = 1; return hipErrorInvalidValue; }
    PrepFwdParams pp{};
    PFwdParams kp{};
    for (int d = 0; d < s.ndir; ++d) {
      pp.hx[d] = sc.buf[d]; pp.h0[d] = dirs[d].h0; pp.bar[d] = sc.bar[d];
      PFwdDir& k = kp.d[d];
      k.zg = dirs[d].zg; k.R = dirs[d].R; k.h0 = dirs[d].h0; k.c0 = dirs[d].c0;
      k.y = dirs[d].y; k.c = dirs[d].c; k.hT = dirs[d].hT; k.cT = dirs[d].cT;
      k.hx = sc.buf[d]; k.bar = sc.bar[d]; k.direction = dirs[d].direction;
    }
    pp.ndir = s.ndir; pp.B = s.B; pp.H = s.H; pp.Bp = pl.Bp; pp.Hp = pl.Hp;
    kp.seq_lens = seq_lens; kp.flag = flag;
    kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy; kp.G = pl.G; kp.Bp = pl.Bp; kp.Hp = pl.Hp;
    hipLaunchKernelGGL(prep_fwd_kernel, dim3(64), dim3(256), 0, stream, pp);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int grid = pl.G * s.ndir;
    const int NT = pl.U / 4;
#define RLSTM_FWD_CASE(MT_, NT_)                                                                      \
    if (pl.MT == MT_ && NT == NT_)                                                                    \
      return coop_launch(lstm_fwd_persistent_kernel<MT_, NT_>, grid, pl.lds_fwd, stream, &kp, resident_err);
    RLSTM_FWD_CASE(1, 1) RLSTM_FWD_CASE(2, 1) RLSTM_FWD_CASE(4, 1)
    RLSTM_FWD_CASE(1, 2) RLSTM_FWD_CASE(2, 2) RLSTM_FWD_CASE(4, 2)
#undef RLSTM_FWD_CASE
    return hipErrorInvalidValue;
  }

  // stepwise
  const size_t bh = (size_t)s.B * s.H;
  SInitParams ip{};
  SFwdParams kp{};
  for (int d = 0; d < s.ndir; ++d) {
    ip.dst[d] = sc.buf[d]; ip.src[d] = dirs[d].h0;
    SFwdDir& k = kp.d[d];
    k.zg = dirs[d].zg; k.R = dirs[d].R; k.c0 = dirs[d].c0; k.y = dirs[d].y; k.c = dirs[d].c;
    k.hT = dirs[d].hT; k.cT = dirs[d].cT; k.hbuf = sc.buf[d]; k.direction = dirs[d].direction;
  }
  ip.ndir = s.ndir; ip.n = bh; ip.off = bh;      // step 0 reads buffer 1
  kp.seq_lens = seq_lens; kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy;
  const unsigned blocks = (unsigned)((bh + 255) / 256);
  hipLaunchKernelGGL(init_state_kernel, dim3(blocks), dim3(256), 0, stream, ip);
  for (int st = 0; st < s.T; ++st) {
    kp.s = st;
    hipLaunchKernelGGL(step_fwd_kernel, dim3(blocks, (unsigned)s.ndir), dim3(256), 0, stream, kp);
  }
  return hipGetLastError();
}

hipError_t rec_backward(hipStream_t stream, const RecShape& s, const RecBwdDir* dirs, const int32_t* seq_lens,
                        void* ws, unsigned* flag, bool persistent, int* resident_err) {
  RecScratch sc = carve(s, ws);
  if (persistent) {
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    PersistentPlan pl = plan_persistent(s, di.num_cus, di.max_lds);
    if (!pl.ok) { *resident_err = 1; return hipErrorInvalidValue; }
    PrepBwdParams pp{};
    PBwdParams kp{};
    for (int d = 0; d < s.ndir; ++d) {
      pp.dzx[d] = sc.buf[d]; pp.bar[d] = sc.bar[d];
      PBwdDir& k = kp.d[d];
      k.zg = dirs[d].zg; k.R = dirs[d].R; k.c = dirs[d].c; k.c0 = dirs[d].c0; k.dy = dirs[d].dy;
      k.dhT = dirs[d].dhT; k.dcT = dirs[d].dcT; k.dh0 = dirs[d].dh0; k.dc0 = dirs[d].dc0; k.db = dirs[d].db;
      k.dzx = sc.buf[d]; k.bar = sc.bar[d]; k.direction = dirs[d].direction;
    }
    pp.ndir = s.ndir; pp.floats = 2 * (size_t)pl.Kp * pl.Bp;
    kp.seq_lens = seq_lens; kp.flag = flag;
    kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy; kp.G = pl.G; kp.Bp = pl.Bp; kp.Kp = pl.Kp;
    hipLaunchKernelGGL(prep_bwd_kernel, dim3(64), dim3(256), 0, stream, pp);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int grid = pl.G * s.ndir;
#define RLSTM_BWD_CASE(MT_, U_)                                                                       \
    if (pl.MT == MT_ && pl.U == U_)                                                                   \
      return coop_launch(lstm_bwd_persistent_kernel<MT_, U_>, grid, pl.lds_bwd, stream, &kp, resident_err);
    RLSTM_BWD_CASE(1, 4) RLSTM_BWD_CASE(2, 4) RLSTM_BWD_CASE(4, 4)
    RLSTM_BWD_CASE(1, 8) RLSTM_BWD_CASE(2, 8) RLSTM_BWD_CASE(4, 8)
#undef RLSTM_BWD_CASE
    return hipErrorInvalidValue;
  }

  // stepwise: buf = [Dh0 | Dh1 | Dc]
  const size_t bh = (size_t)s.B * s.H;
  SInitParams ih{}, ic{};
  SBwdParams kp{};
  for (int d = 0; d < s.ndir; ++d) {
    ih.dst[d] = sc.buf[d]; ih.src[d] = dirs[d].dhT;
    ic.dst[d] = sc.buf[d]; ic.src[d] = dirs[d].dcT;
    SBwdDir& k = kp.d[d];
    k.zg = dirs[d].zg; k.R = dirs[d].R; k.c = dirs[d].c; k.c0 = dirs[d].c0; k.dy = dirs[d].dy;
    k.dh0 = dirs[d].dh0; k.dc0 = dirs[d].dc0;
    k.dhbuf = sc.buf[d]; k.dcbuf = sc.buf[d] + 2 * bh; k.direction = dirs[d].direction;
  }
  ih.ndir = ic.ndir = s.ndir; ih.n = ic.n = bh; ih.off = bh; ic.off = 2 * bh;
  kp.seq_lens = seq_lens; kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy;
  const unsigned blocks = (unsigned)((bh + 255) / 256);
  hipLaunchKernelGGL(init_state_kernel, dim3(blocks), dim3(256), 0, stream, ih);
  hipLaunchKernelGGL(init_state_kernel, dim3(blocks), dim3(256), 0, stream, ic);
  for (int st = 0; st < s.T; ++st) {
    kp.s = st;
    hipLaunchKernelGGL(step_bwd_gates_kernel, dim3(blocks, (unsigned)s.ndir), dim3(256), 0, stream, kp);
    hipLaunchKernelGGL(step_bwd_dh_kernel, dim3(blocks, (unsigned)s.ndir), dim3(256), 0, stream, kp);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  for (int d = 0; d < s.ndir; ++d) {
    e = column_sum(stream, dirs[d].zg, (size_t)s.T * s.B, 4 * s.H, 4 * s.H, dirs[d].db);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace rlstm
