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
// loads only, never through plain cached accesses:
//   * h_t and d a_t: the producer stores its values, waits until the stores
//     are acknowledged (s_waitcnt vmcnt(0)), then raises its own step flag;
//     a consumer wavefront polls only the flags of the producers whose rows it
//     multiplies, then fetches those rows with 16-byte device-scope buffer
//     loads, all issued before the first MFMA.  The exchange arrays are laid
//     out in MFMA operand order so each such load is a contiguous 1 KiB per
//     wavefront.  Buffers are double-buffered by step parity.
//   * partial tiles: every value travels as one 64-bit word (value, step tag),
//     so the consumer polls the data itself and no flag round trip is needed.
// There is no device-wide barrier and no cache write-back / invalidate in the
// step loop.  All waits are bounded: on expiry the kernel raises the timeout
// flag and every workgroup leaves its loop.
//
// Three forms of the recurrent product (template argument PREC of the kernels):
// 0 fp32 values on the fp32 matrix instructions (as described above); 1 values
// rounded to bf16 (operand_dtype 1: v_mfma_f32_16x16x32_bf16, R and the
// exchanged rows at 2 bytes per value); 2 fp32 values as three bf16 parts each
// (groups of more than 16 sequences: six bf16 instructions per product, see
// wave_product_3).  Everything outside the product is fp32 in all three.
#include "rlstm_internal.h"

namespace rlstm {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr unsigned long long kDefaultWaitTicks = 400000000ull;   // 4 s of the 100 MHz wall clock
// 16-byte loads in flight per lane: a multiple of the batch tiles MT, so that a group of loads starts at a whole k-step.
// Three row tiles (the 48-row kernels, which run with nothing beside them and can afford the registers) fetch all 24
// chunks of a 512-unit layer at once: a second group of loads would add a second load latency to every step.
template <int MT> constexpr int load_group() { return MT == 3 ? 24 : 16; }
constexpr int kAuxSc1 = 16;             // buffer-load cache policy: device scope

// ---- bounded spinning --------------------------------------------------------
struct Spin {
  unsigned n = 0;
  unsigned long long t0 = 0;
  unsigned long long limit;
  __device__ __forceinline__ explicit Spin(unsigned long long wait_ticks) : limit(wait_ticks) {}
  // call once per unsuccessful poll; true = give up
  __device__ __forceinline__ bool expired(unsigned* err) {
    if ((++n & 1023u) != 0) return false;
    const unsigned long long now = wall_clock64();
    if (t0 == 0) { t0 = now; return false; }
    if (now - t0 > limit) return true;
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

// Step flags.  Every producer keeps kFlagCopies copies of its flag, each copy set in its own
// 4 KiB block, and a consumer workgroup polls copy (its index mod kFlagCopies): polls of one
// memory line by many wavefronts are served one after the other, so with a single copy the
// ~125 pollers of each line would queue behind each other for microseconds.
constexpr int kFlagCopies = 64;
constexpr int kFlagCopyStride = 1024;            // unsigned words between copies

__device__ __forceinline__ void publish_flag(unsigned* flags, int wg, unsigned value) {
  if (threadIdx.x < kFlagCopies) st_dev(flags + threadIdx.x * kFlagCopyStride + wg, value);
}

// Test hook against races in the exchange: workgroup `slow_wg` holds back what it is about to publish (data, then flag)
// for `ticks` of the 100 MHz wall clock, every step.  A consumer that read an exchange buffer without having waited for
// its producer would then read the values of two steps ago, and the results would differ from an undisturbed run; a
// correct kernel gives the same bits, only later.  The wait is bounded by `ticks` (the host limits it to 1 ms).
__device__ __forceinline__ void test_delay(int slow_wg, unsigned ticks) {
  if ((int)blockIdx.x != slow_wg || ticks == 0u) return;
  const unsigned long long t0 = wall_clock64();
  while (wall_clock64() - t0 < (unsigned long long)ticks) __builtin_amdgcn_s_sleep(4);
}

// A wavefront waits until flags[first .. first+count) (clipped to limit) have all reached `want`.
__device__ __forceinline__ bool wave_wait_flags(const unsigned* flags, int first, int count, int limit,
                                                unsigned want, unsigned* err, unsigned long long wait_ticks) {
  const int lane = threadIdx.x & 63;
  const bool mine = lane < count && first + lane < limit;
  const unsigned* src = flags + (mine ? first + lane : first);
  Spin sp(wait_ticks);
  bool ok = true;
  for (;;) {
    const bool ready = !mine || ld_dev(src) >= want;
    if (__all(ready)) break;
    if (sp.expired(err)) { ok = false; break; }
  }
  compiler_fence();
  return ok;
}

// Workgroup barrier that also tells every thread whether any thread failed (a bounded wait expired).  `flag` is a
// word of LDS that starts at zero and is only ever raised; two successive uses need two different words, or a
// plain barrier between them.  (__syncthreads_or costs three barriers.)
__device__ __forceinline__ bool barrier_any_failed(int fail, int* flag) {
  if (fail) *flag = 1;
  __syncthreads();
  return *flag != 0;
}

// gate functions on the hardware exponential (v_exp_f32, 1 ulp) and reciprocal (v_rcp_f32, 1 ulp): the gating sits in
// the step chain, and the libm expf is a dozen instructions longer per call.  Absolute error ~2e-7.
__device__ __forceinline__ float fexp(float u) { return __builtin_amdgcn_exp2f(u * 1.44269504088896341f); }
__device__ __forceinline__ float fsigmoid(float u) { return __builtin_amdgcn_rcpf(1.0f + fexp(-u)); }
__device__ __forceinline__ float ftanh(float u) { return 2.0f * __builtin_amdgcn_rcpf(1.0f + fexp(-2.0f * u)) - 1.0f; }

// position of element (row k of a wavefront's K range, sequence b) inside that wavefront's
// operand-ordered block: [chunk][lane][4], L = (k/4)*MT + b/16, chunk = L/4, lane = (k%4)*16 + b%16
template <int MT>
__device__ __forceinline__ int operand_slot(int k, int b) {
  const int L = (k >> 2) * MT + (b >> 4);
  return ((L >> 2) * 64 + (k & 3) * 16 + (b & 15)) * 4 + (L & 3);
}

// column of the resident fp32 matrix in LDS: row k keeps its 16*NT columns rotated by 16*(k%4), so
// that the four rows one MFMA operand fetch touches fall into different banks
template <int NT>
__device__ __forceinline__ int rotated_col(int k, int col) { return (col + 16 * (k & 3)) & (16 * NT - 1); }

// One wavefront's share of a [B x K] * [K x 16*NT] product.  A rows come from the exchange
// array (device-scope 16-byte loads, operand order), B rows from LDS (row stride 16*NT floats,
// columns rotated per row).  HALF: only sequences 0..7 of the tile exist; the other lanes load nothing.
template <int MT, int NT, bool HALF>
__device__ __forceinline__ void wave_product(const float* xblock, int xblock_bytes, int nch, const float* bs,
                                             floatx4 (&acc)[MT][NT]) {
  constexpr int ldb = 16 * NT;
  const int lane = threadIdx.x & 63, l16 = lane & 15, lq = lane >> 4;
  const bool loads = !HALF || l16 < 8;
  __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(xblock), 0, xblock_bytes, 0x00020000);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  constexpr int CG = load_group<MT>();
  for (int c0 = 0; c0 < nch; c0 += CG) {
    floatx4 v[CG];
#pragma unroll
    for (int q = 0; q < CG; ++q) {
      v[q] = floatx4{0.f, 0.f, 0.f, 0.f};
      if (loads)
        v[q] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, ((c0 + q) * 64 + lane) * 16, 0, kAuxSc1));
    }
    // chunks past nch read beyond the buffer resource's size and return zeros; their MFMAs are skipped
#pragma unroll
    for (int q = 0; q < CG; ++q) {
      if (c0 + q < nch) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          // element w of chunk c0 + q is pair L = (c0 + q) * 4 + w of the (k-step, batch tile) sequence;
          // 4 * CG is a multiple of MT, so the tile index does not depend on c0
          const int ks = (c0 * 4) / MT + (q * 4 + w) / MT;
          const int mt = (q * 4 + w) % MT;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const float bf = bs[(ks * 4 + lq) * ldb + ((nt + lq) & (NT - 1)) * 16 + l16];
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(v[q][w], bf, acc[mt][nt], 0, 0, 0);
          }
        }
      }
    }
  }
}

// ---- bf16-operand variant (operand_dtype = 1): the exchanged h_t / d a_t and the resident R / R^T are
// bf16 (round to nearest even), products accumulate in fp32 (v_mfma_f32_16x16x32_bf16), everything else
// stays fp32.  A lane's MFMA operand is 8 consecutive k of one row, i.e. one 16-byte chunk.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ unsigned short bf16_bits(float v) { return __builtin_bit_cast(unsigned short, (__bf16)v); }

// position (in bf16 elements) of (row kr of a wavefront's K range, sequence b) inside that wavefront's
// operand-ordered block: [chunk = (kr/32)*MT + b/16][lane = ((kr%32)/8)*16 + b%16][kr%8]
template <int MT>
__device__ __forceinline__ int operand_slot_bf(int kr, int b) {
  const int chunk = (kr >> 5) * MT + (b >> 4);
  return (chunk * 64 + ((kr >> 3) & 3) * 16 + (b & 15)) * 8 + (kr & 7);
}

// B rows in LDS: [k/8][ldn columns][8] bf16
// ROLL: how a K range of more than CG chunks is fetched, see below (measured per kernel)
template <int MT, int NT, bool HALF, bool ROLL>
__device__ __forceinline__ void wave_product_bf(const void* xblock, int xblock_bytes, int nch, const unsigned short* bs,
                                                floatx4 (&acc)[MT][NT]) {
  constexpr int ldn = 16 * NT;
  const int lane = threadIdx.x & 63, l16 = lane & 15, lq = lane >> 4;
  const bool loads = !HALF || l16 < 8;
  __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(xblock), 0, xblock_bytes, 0x00020000);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  constexpr int CG = load_group<MT>();
  // How a K range of more than CG chunks is fetched.  !ROLL: in groups of CG loads, each group in registers of its own
  // (the next group is requested when the MFMAs of the last one are issued).  ROLL: a window of CG loads stays in
  // flight; as soon as a chunk's MFMAs are issued, its registers take the chunk CG further on, so that the range is
  // one continuous stream of loads.  At 6 x 1000 units, 64 sequences (32 chunks per wavefront) the window makes the
  // backward step 1.1 us shorter (9.9 against 11.0) and the forward step 0.7 us longer (7.3 against 6.6; also in a
  // form that reuses one group's registers for the next group; groups or a window of 24: 7.0 / 8.8), so each kernel
  // takes the form that suits it.  Up to CG chunks both are the same.
  if constexpr (!ROLL) {
    for (int c0 = 0; c0 < nch; c0 += CG) {
      intx4 v[CG];
#pragma unroll
      for (int q = 0; q < CG; ++q) {
        v[q] = intx4{0, 0, 0, 0};
        if (loads) v[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, ((c0 + q) * 64 + lane) * 16, 0, kAuxSc1);
      }
#pragma unroll
      for (int q = 0; q < CG; ++q) {
        if (c0 + q < nch) {
          const int ks = (c0 + q) / MT;              // CG is a multiple of MT, so q % MT is the batch tile
          const int mt = q % MT;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(bs + ((size_t)(ks * 4 + lq) * ldn + nt * 16 + l16) * 8);
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v[q]), bfrag, acc[mt][nt], 0, 0, 0);
          }
        }
      }
    }
  } else {
    intx4 v[CG];
#pragma unroll
    for (int q = 0; q < CG; ++q) {
      v[q] = intx4{0, 0, 0, 0};
      if (loads && q < nch) v[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (q * 64 + lane) * 16, 0, kAuxSc1);
    }
    for (int c0 = 0; c0 < nch; c0 += CG) {
#pragma unroll
      for (int q = 0; q < CG; ++q) {
        if (c0 + q < nch) {
          const int ks = (c0 + q) / MT;
          const int mt = q % MT;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(bs + ((size_t)(ks * 4 + lq) * ldn + nt * 16 + l16) * 8);
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v[q]), bfrag, acc[mt][nt], 0, 0, 0);
          }
        }
        if (c0 + CG + q < nch) {
          v[q] = intx4{0, 0, 0, 0};
          if (loads) v[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, ((c0 + CG + q) * 64 + lane) * 16, 0, kAuxSc1);
        }
      }
    }
  }
}

// ---- three-part variant (fp32 operands, groups of more than 16 sequences): the exchanged h_t / d a_t and the
// resident R / R^T are each kept as THREE bf16 parts that add up to the fp32 value exactly (its 24 significant bits
// cut 8 + 8 + 8), and the product is the sum of the six largest of the nine part products, as in the large matrix
// products (gemm_f32_3xbf16_kernel): 6 v_mfma_f32_16x16x32_bf16 do the work of 8 v_mfma_f32_16x16x4_f32 in 3/8 of
// the matrix cores' time; what is left out is below 2^-21 of each term.  With two or three 16-row tiles per workgroup
// the matrix instructions are a third of the step, which is where this pays; with one tile the 1.5 x larger
// exchange costs what the shorter instructions save, and the fp32 kernels stay.
// Layouts: as the bf16 variant, once per part - a wavefront's exchange block is [part][chunk][lane][16 bytes], the
// resident matrix [part][k/8][columns][8].
__device__ __forceinline__ void cut3_bits(float x, unsigned& b1, unsigned& b2, unsigned& b3) {
  const unsigned a1 = __float_as_uint(x) & 0xffff0000u;
  const float r = x - __uint_as_float(a1);                    // exact
  const unsigned a2 = __float_as_uint(r) & 0xffff0000u;
  const float r2 = r - __uint_as_float(a2);                   // exact, at most 8 significant bits
  b1 = a1 >> 16; b2 = a2 >> 16; b3 = __float_as_uint(r2) >> 16;
}

// nchp: chunks per part; bplane: bf16 elements between the parts of the resident matrix.  All chunks of a K range of
// up to 4 k-steps (a quarter of 512 units) are requested at once, 3 * 4 * MT of them.
template <int MT, int NT>
__device__ __forceinline__ void wave_product_3(const void* xblock, int xblock_bytes, int nchp, const unsigned short* bs,
                                               int bplane, floatx4 (&acc)[MT][NT]) {
  constexpr int ldn = 16 * NT;
  constexpr int KG = 4;                            // k-steps per group of loads
  const int lane = threadIdx.x & 63, l16 = lane & 15, lq = lane >> 4;
  __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(xblock), 0, xblock_bytes, 0x00020000);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  const int nks = nchp / MT;
  for (int k0 = 0; k0 < nks; k0 += KG) {
    intx4 v[3][KG * MT];
#pragma unroll
    for (int part = 0; part < 3; ++part)
#pragma unroll
      for (int q = 0; q < KG * MT; ++q) {
        // a chunk past the part's last one is given an offset beyond the block and reads zeros
        const int c = k0 * MT + q;
        const unsigned off = c < nchp ? (unsigned)(((part * nchp + c) * 64 + lane) * 16) : 0x80000000u;
        v[part][q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, kAuxSc1);
      }
#pragma unroll
    for (int kk = 0; kk < KG; ++kk) {
      const int ks = k0 + kk;
      if (ks < nks) {
        bf16x8 bfrag[3][NT];
#pragma unroll
        for (int part = 0; part < 3; ++part)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            bfrag[part][nt] = *reinterpret_cast<const bf16x8*>(bs + (size_t)part * bplane + ((size_t)(ks * 4 + lq) * ldn + nt * 16 + l16) * 8);
        // small terms first; the tiles alternate so that no instruction waits for the one before it
        constexpr int QA[6] = {2, 0, 1, 1, 0, 0}, QB[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
        for (int t = 0; t < 6; ++t)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v[QA[t]][kk * MT + mt]), bfrag[QB[t]][nt],
                                                                   acc[mt][nt], 0, 0, 0);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------
// Workgroups form NG = ndir * nb groups: group g runs direction g % ndir for the sequences
// [(g / ndir) * Bg, + Bg) and exchanges data only among its own members.  Workgroup index =
// member * NG + g: the dispatcher deals consecutive workgroups out to the 8 XCDs in turn, so with
// NG = 8 a group sits on one XCD (with NG = 4 on two), whose L2 then serves the group's exchange.
constexpr int kMaxGroups = 8;
struct PFwdDir {
  float* zg; const float* R; const float* h0; const float* c0;
  float* y; float* c; float* hT; float* cT;
  float* hstate; float* cstate;   // [B,H] each: carried state between launches that split the T steps
  int direction;
};
struct PFwdParams {
  PFwdDir d[2];
  void* hx[kMaxGroups];            // per group: 2 x [4 wavefronts][nch][64][16 bytes]
  unsigned* flags[kMaxGroups];     // per group: [flag copies][Gf]
  int ndir, NG, Bg;
  const int32_t* seq_lens;
  unsigned* err;
  unsigned long long wait_ticks;   // bound of every wait, in 100 MHz wall-clock ticks
  int mute_wg;                     // test hook: this workgroup withholds its step flags (-1: none)
  int slow_wg; unsigned slow_ticks; // test hook: this workgroup publishes every step late (see test_delay)
  int T, B, H, ldy, Gf, Hp, nch;
  int s_begin, s_end;              // steps [s_begin, s_end) of the T steps are done by this launch
};

// Workgroup = 4 compute wavefronts (threads 0..255) + 1 I/O wavefront (threads 256..319).
// The compute wavefronts touch global memory only through the device-scope exchange; the I/O
// wavefront moves the frame's input part from HBM into LDS one step ahead and the frame's
// outputs (gates, y, c) from LDS to HBM one step behind, so HBM latency and store
// acknowledgements never sit in the step's dependency chain.
constexpr int kBlockThreads = 320;

// ROWS: sequences a group can hold (8, 16, 32, 48 or 64); 8 uses half of one 16-row MFMA tile.
// PREC: 0 fp32 matrix instructions, 1 operands rounded to bf16, 2 fp32 operands as three bf16 parts
template <int ROWS, int NT, int PREC>
__global__ __launch_bounds__(kBlockThreads) void lstm_fwd_persistent_kernel(PFwdParams p) {
  constexpr bool BF = PREC == 1, P3 = PREC == 2;
  constexpr int MT = ROWS <= 16 ? 1 : ROWS / 16;
  constexpr bool HALF = ROWS == 8;
  constexpr int U = 4 * NT, NC = 16 * NT;
  constexpr int NE = ROWS * U;                   // (sequence, unit) pairs of this workgroup (multiple of 64)
  constexpr int EPT = (NE + 255) / 256;          // pairs per compute thread
  constexpr int EPL = NE / 64;                   // pairs per I/O lane
  static_assert(NE % 64 == 0, "pairs must fill whole I/O wavefronts");
  extern __shared__ __align__(16) float lds[];
  const int grp = blockIdx.x % p.NG, wg = blockIdx.x / p.NG;
  const int dir = grp % p.ndir, b0 = (grp / p.ndir) * p.Bg;
  const PFwdDir& D = p.d[dir];
  const int T = p.T, H = p.H, Hp = p.Hp, nch = p.nch;
  const int B = min(p.Bg, p.B - b0);             // sequences of this group (local index 0 .. B-1, global b0 + index)
  if (B <= 0) return;                            // a group without sequences: all its workgroups leave
  const int s_begin = p.s_begin, s_end = p.s_end;
  // an earlier launch of this pass gave up waiting: the exchange arrays are not valid, do nothing
  if (ld_dev(p.err) != 0u) return;
  // the step chain is latency-bound: its wavefronts go before those of any kernel sharing the CU
  __builtin_amdgcn_s_setprio(3);
  const int u0 = wg * U;
  float* Rs = lds;                               // fp32: [Hp][NC]; bf16: [Hp/8][NC][8] (half the size); three parts: 3 of those
  unsigned short* Rsb = reinterpret_cast<unsigned short*>(lds);
  float* Red = Rs + (size_t)Hp * NC * (P3 ? 3 : (BF ? 1 : 2)) / 2;   // [4][MT][NT][256]
  float* zin = Red + 4 * MT * NT * 256;          // [2][4][NE]  input part of the frame, per gate
  float* gout = zin + 2 * 4 * NE;                // [2][6][NE]  gates i,f,o,g, y, c of the frame
  int* failed = reinterpret_cast<int*>(gout + 2 * 6 * NE);   // raised when a bounded wait expired

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wavefront-uniform, kept in a scalar register
  const bool is_io = wave == 4;
  const int lane = tid & 63;

  // resident slice of R: slice column g*U + uu is column g*H + u0 + uu of R
  for (int idx = tid; idx < Hp * NC; idx += kBlockThreads) {
    const int k = idx / NC, col = idx % NC;
    const int g = col / U, u = u0 + col % U;
    const float v = (k < H && u < H) ? D.R[(size_t)k * 4 * H + g * H + u] : 0.f;
    if (P3) {
      unsigned b1, b2, b3;
      cut3_bits(v, b1, b2, b3);
      unsigned short* q = Rsb + ((size_t)(k >> 3) * NC + col) * 8 + (k & 7);
      q[0] = (unsigned short)b1; q[(size_t)Hp * NC] = (unsigned short)b2; q[(size_t)2 * Hp * NC] = (unsigned short)b3;
    } else if (BF) Rsb[((size_t)(k >> 3) * NC + col) * 8 + (k & 7)] = bf16_bits(v);
    else Rs[k * NC + rotated_col<NT>(k, col)] = v;
  }

  const int KW = Hp / 4;                         // rows of h per wavefront
  const int nchp = nch / 3;                      // three parts: chunks per part
  const int wbytes = nch * 1024;                 // bytes of one wavefront's operand block (64 lanes x 16 bytes per chunk)
  const size_t hxsz = (size_t)4 * wbytes;        // bytes of one step buffer
  char* const hxbase = static_cast<char*>(p.hx[grp]);
  unsigned* const gflags = p.flags[grp];

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
      const size_t bu = (size_t)(b0 + eb[e]) * H + eu[e];
      if (s_begin > 0) { hreg[e] = D.hstate[bu]; creg[e] = D.cstate[bu]; }
      else {
        if (D.h0) hreg[e] = D.h0[bu];
        if (D.c0) creg[e] = D.c0[bu];
      }
      elen[e] = min(max(p.seq_lens[b0 + eb[e]], 0), T);
      eslot[e] = (BF || P3) ? (eu[e] / KW) * (wbytes / 2) + operand_slot_bf<MT>(eu[e] % KW, eb[e])
                            : (eu[e] / KW) * (wbytes / 4) + operand_slot<MT>(eu[e] % KW, eb[e]);
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
        zr[i][g] = iv[i] ? D.zg[((size_t)t * p.B + b0 + ib[i]) * 4 * H + g * H + iu[i]] : 0.f;
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
      const size_t row = (size_t)t * p.B + b0 + ib[i];
      float* zrow = D.zg + row * 4 * H + iu[i];
      zrow[0] = src[0 * NE + j]; zrow[H] = src[1 * NE + j]; zrow[2 * H] = src[2 * NE + j]; zrow[3 * H] = src[3 * NE + j];
      D.y[row * p.ldy + iu[i]] = src[4 * NE + j];
      D.c[row * H + iu[i]] = src[5 * NE + j];
    }
  };
  if (is_io) {
    io_load(s_begin);
    io_stage(s_begin);
    if (s_begin + 1 < s_end) io_load(s_begin + 1);
  }
  if (tid == 0) *failed = 0;
  __syncthreads();

  const int prod_first = wave * KW / U, prod_count = KW / U;
  const unsigned* myflags = gflags + (wg % kFlagCopies) * kFlagCopyStride;

  // Step s reads the h that step s-1 left in the exchange array, also when step s-1 was the last
  // step of the previous launch: flags, exchange arrays and tags live in device memory.
  for (int s = s_begin; s < s_end; ++s) {
    const int t = D.direction > 0 ? s : T - 1 - s;
    const char* hprev = hxbase + (size_t)((s + 1) & 1) * hxsz;
    char* hcur = hxbase + (size_t)(s & 1) * hxsz;
    int fail = 0;

    if (!is_io) {
      // h of the previous step: wait for the producers of this wavefront's rows, then h_prev * R
      if (s > 0 && !wave_wait_flags(myflags, prod_first, prod_count, p.Gf, (unsigned)s, p.err, p.wait_ticks)) fail = 1;
      floatx4 acc[MT][NT];
      if (P3) wave_product_3<MT, NT>(hprev + (size_t)wave * wbytes, wbytes, nchp, Rsb + (size_t)wave * KW * NC, Hp * NC, acc);
      else if (BF) wave_product_bf<MT, NT, HALF, false>(hprev + (size_t)wave * wbytes, wbytes, nch, Rsb + (size_t)wave * KW * NC, acc);
      else wave_product<MT, NT, HALF>(reinterpret_cast<const float*>(hprev + (size_t)wave * wbytes), wbytes, nch,
                                      Rs + (size_t)wave * KW * NC, acc);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          *reinterpret_cast<floatx4*>(Red + ((wave * MT + mt) * NT + nt) * 256 + lane * 4) = acc[mt][nt];
    } else {
      // stage the next frame's input part (loaded a step ago), write out the previous frame's
      // outputs, start loading the frame after next: every wait here is on work issued a step ago
      if (s + 1 < s_end) io_stage(s + 1);
      if (s > s_begin) io_store(s - 1);
      if (s + 2 < s_end) io_load(s + 2);
    }
    if (barrier_any_failed(fail, failed)) {      // the plain barrier further down separates this use from the next
      if (tid == 0) st_dev(p.err, 1u);
      return;
    }

    if (!is_io) {
      // gating, cell update, mask; publish the carried h; leave the frame's outputs in LDS
      test_delay(p.slow_wg, p.slow_ticks);
      const float* zcur = zin + (s & 1) * 4 * NE;
      float* ocur = gout + (s & 1) * 6 * NE;
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        if (BF) {
          // (handled after the loop: bf16 values are published in pairs)
        }
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
        if (!BF && !P3) st_dev(reinterpret_cast<float*>(hcur) + eslot[e], hreg[e]);
        ocur[0 * NE + j] = gi; ocur[1 * NE + j] = gf; ocur[2 * NE + j] = go; ocur[3 * NE + j] = gg;
        ocur[4 * NE + j] = valid ? hn : 0.f;
        ocur[5 * NE + j] = creg[e];
      }
      if (BF) {
        // units u, u+1 (u even) are neighbouring lanes and neighbouring bf16 slots: publish them as one word
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
          const unsigned mine = ev[e] ? bf16_bits(hreg[e]) : 0u;
          const unsigned other = __shfl_xor(mine, 1);
          if (ev[e] && !(eu[e] & 1))
            st_dev(reinterpret_cast<unsigned*>(hcur) + (eslot[e] >> 1), mine | (other << 16));
        }
      }
      if (P3) {
        // the same pairs, once per part (a part's chunks are nchp * 1024 bytes on)
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
          unsigned m1 = 0u, m2 = 0u, m3 = 0u;
          if (ev[e]) cut3_bits(hreg[e], m1, m2, m3);
          const unsigned o1 = __shfl_xor(m1, 1), o2 = __shfl_xor(m2, 1), o3 = __shfl_xor(m3, 1);
          if (ev[e] && !(eu[e] & 1)) {
            unsigned* dst = reinterpret_cast<unsigned*>(hcur) + (eslot[e] >> 1);
            st_dev(dst, m1 | (o1 << 16));
            st_dev(dst + nchp * 256, m2 | (o2 << 16));
            st_dev(dst + 2 * nchp * 256, m3 | (o3 << 16));
          }
        }
      }
      wait_stores_acked();
    }
    __syncthreads();
    if ((int)blockIdx.x != p.mute_wg) publish_flag(gflags, wg, (unsigned)(s + 1));

  }
  __syncthreads();
  if (is_io) io_store(s_end - 1);

#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    if (!ev[e]) continue;
    const size_t bu = (size_t)(b0 + eb[e]) * H + eu[e];
    if (s_end < T) { D.hstate[bu] = hreg[e]; D.cstate[bu] = creg[e]; }
    else {
      if (D.hT) D.hT[bu] = hreg[e];
      if (D.cT) D.cT[bu] = creg[e];
    }
  }
}

// ---------------------------------------------------------------------------
// backward
// ---------------------------------------------------------------------------
struct PBwdDir {
  float* zg; const float* R; const float* c; const float* c0; const float* dy;
  const float* dhT; const float* dcT; float* dh0; float* dc0; float* db;
  float* dhstate; float* dcstate;   // [B,H] each: carried gradients between launches that split the T steps
  float* dbpart;                    // [nb][4H]: bias gradient of each group of sequences (summed afterwards)
  int direction;
};
struct PBwdParams {
  PBwdDir d[2];
  void* dzx[kMaxGroups];                  // per group: 2 x [4 quarters][4 wavefronts][nch][64][16 bytes]
  unsigned long long* part[kMaxGroups];   // per group: 2 x [PG][4][Bp][UG] (value, tag)
  unsigned* flags[kMaxGroups];            // per group: [flag copies][Gb]
  int ndir, NG, Bg;
  const int32_t* seq_lens;
  unsigned* err;
  unsigned long long wait_ticks;
  int mute_wg;
  int slow_wg; unsigned slow_ticks;
  int T, B, H, ldy, PG, Hq, nch;
  int s_begin, s_end;
};

// Same workgroup shape as the forward kernel: 4 compute wavefronts + 1 I/O wavefront that stages
// the frame's gates, cell states and dy from HBM into LDS one step ahead and writes d a back to
// HBM one step behind.
template <int ROWS, int NT, int PREC>
__global__ __launch_bounds__(kBlockThreads) void lstm_bwd_persistent_kernel(PBwdParams p) {
  constexpr bool BF = PREC == 1, P3 = PREC == 2;
  constexpr int MT = ROWS <= 16 ? 1 : ROWS / 16;
  constexpr bool HALF = ROWS == 8;
  constexpr int U = 4 * NT, UG = 16 * NT, Bp = 16 * MT;
  constexpr int NE = ROWS * U;                   // (sequence, unit) pairs owned by this workgroup
  constexpr int EPT = (NE + 255) / 256;
  constexpr int EPL = NE / 64;
  static_assert(NE % 64 == 0, "pairs must fill whole I/O wavefronts");
  extern __shared__ __align__(16) float lds[];
  const int Gb = 4 * p.PG;
  const int grp = blockIdx.x % p.NG, wg = blockIdx.x / p.NG;
  const int dir = grp % p.ndir, bgi = grp / p.ndir, b0 = bgi * p.Bg;
  const int pg = wg >> 2, qq = wg & 3;           // unit group, K quarter (also: which quarter of the group it owns)
  const PBwdDir& D = p.d[dir];
  const int T = p.T, H = p.H, Hq = p.Hq, nch = p.nch;
  const int B = min(p.Bg, p.B - b0);             // sequences of this group (local index; global b0 + index)
  if (B <= 0) return;
  const int s_begin = p.s_begin, s_end = p.s_end;
  if (ld_dev(p.err) != 0u) return;               // an earlier launch of this pass gave up waiting
  __builtin_amdgcn_s_setprio(3);                 // latency-bound chain: ahead of any kernel sharing the CU
  const int u0 = wg * U;                         // owned units
  float* RTs = lds;                              // fp32: [4*Hq][UG]; bf16: [4*Hq/8][UG][8] (half the size)
  unsigned short* RTb = reinterpret_cast<unsigned short*>(lds);
  float* Red = RTs + (size_t)4 * Hq * UG * (P3 ? 3 : (BF ? 1 : 2)) / 2;   // [4][MT][NT][256]
  float* bin = Red + 4 * MT * NT * 256;          // [2][7][NE]  gates i,f,o,g, c, c_prev, dy of the frame
  float* dzo = bin + 2 * 7 * NE;                 // [2][4][NE]  d a of the frame
  int* failed = reinterpret_cast<int*>(dzo + 2 * 4 * NE);   // two words raised when a bounded wait expired

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wavefront-uniform, kept in a scalar register
  const bool is_io = wave == 4;
  const int lane = tid & 63;
  const int UW = Hq / 4;                         // units per wavefront of a quarter
  // Quarters that hold no unit (small H) contribute nothing: their workgroups publish no partial
  // tile and owners do not wait for one.  Every workgroup that does publish is paced by the flags
  // of real producers, so no tile is overwritten before its owners have read it.
  const int nq = (H + Hq - 1) / Hq;

  // resident rows of R^T: row r = (wavefront w, unit ur of it, gate g) -> unit uk = qq*Hq + w*UW + ur;
  // RTs[r][n] = R[pg*UG + n][g*H + uk]
  for (int idx = tid; idx < 4 * Hq * UG; idx += kBlockThreads) {
    const int r = idx / UG, n = idx % UG;
    const int w = r / Hq, rr = r % Hq;
    const int uk = qq * Hq + w * UW + (rr >> 2), g = rr & 3;
    const int un = pg * UG + n;
    const float v = (uk < H && un < H) ? D.R[(size_t)un * 4 * H + g * H + uk] : 0.f;
    if (P3) {
      unsigned b1, b2, b3;
      cut3_bits(v, b1, b2, b3);
      unsigned short* q = RTb + ((size_t)(r >> 3) * UG + n) * 8 + (r & 7);
      q[0] = (unsigned short)b1; q[(size_t)4 * Hq * UG] = (unsigned short)b2; q[(size_t)8 * Hq * UG] = (unsigned short)b3;
    } else if (BF) RTb[((size_t)(r >> 3) * UG + n) * 8 + (r & 7)] = bf16_bits(v);
    else RTs[r * UG + rotated_col<NT>(r, n)] = v;
  }

  const int nchp = nch / 3;                      // three parts: chunks per part
  const int wbytes = nch * 1024;                 // bytes per (quarter, wavefront) operand block
  const size_t xsz = (size_t)16 * wbytes;        // bytes of one step buffer
  char* const dzbase = static_cast<char*>(p.dzx[grp]);
  unsigned long long* const gpart = p.part[grp];
  unsigned* const gflags = p.flags[grp];
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
      const size_t bu = (size_t)(b0 + eb[e]) * H + eu[e];
      elen[e] = min(max(p.seq_lens[b0 + eb[e]], 0), T);
      if (s_begin > 0) {
        Dh[e] = D.dhstate[bu]; Dc[e] = D.dcstate[bu];
        const int tlast = D.direction > 0 ? T - s_begin : s_begin - 1;   // frame of step s_begin - 1
        vprev[e] = tlast < elen[e];
      } else {
        if (D.dhT) Dh[e] = D.dhT[bu];
        if (D.dcT) Dc[e] = D.dcT[bu];
      }
      // d a of unit u, gate g sits in quarter u/Hq, wavefront (u%Hq)/UW, row ((u%Hq)%UW)*4 + g
      const int ul = eu[e] % Hq;
      eslot[e] = (BF || P3) ? ((eu[e] / Hq) * 4 + ul / UW) * (wbytes / 2) + operand_slot_bf<MT>((ul % UW) * 4, eb[e])
                            : ((eu[e] / Hq) * 4 + ul / UW) * (wbytes / 4) + operand_slot<MT>((ul % UW) * 4, eb[e]);
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
      const size_t row = (size_t)t * p.B + b0 + ib[i];
      const float* zrow = D.zg + row * 4 * H + iu[i];
      lr[i][0] = zrow[0]; lr[i][1] = zrow[H]; lr[i][2] = zrow[2 * H]; lr[i][3] = zrow[3 * H];
      if (tprev >= 0 && tprev < T) lr[i][4] = D.c[((size_t)tprev * p.B + b0 + ib[i]) * H + iu[i]];
      else lr[i][4] = D.c0 ? D.c0[(size_t)(b0 + ib[i]) * H + iu[i]] : 0.f;
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
      float* zrow = D.zg + ((size_t)t * p.B + b0 + ib[i]) * 4 * H + iu[i];
      zrow[0] = src[0 * NE + j]; zrow[H] = src[1 * NE + j]; zrow[2 * H] = src[2 * NE + j]; zrow[3 * H] = src[3 * NE + j];
    }
  };
  if (is_io) {
    const int t0 = frame_of(s_begin);
#pragma unroll
    for (int i = 0; i < EPL; ++i)
      if (iv[i]) cnext[i] = D.c[((size_t)t0 * p.B + b0 + ib[i]) * H + iu[i]];
    io_load(s_begin);
    io_stage(s_begin);
    if (s_begin + 1 < s_end) io_load(s_begin + 1);
  }
  if (tid < 2) failed[tid] = 0;
  __syncthreads();

  // producers of this wavefront's rows: owners of units [qq*Hq + wave*UW, +UW)
  const int prod_first = (qq * Hq + wave * UW) / U, prod_count = UW / U;
  const unsigned* myflags = gflags + (wg % kFlagCopies) * kFlagCopyStride;

  // sums the partial tiles of step `step` for the owned pairs (tag = step + 1).  The words of all owned pairs are
  // requested together and checked together: one round trip through the memory side per poll, however many pairs a
  // thread owns.
  auto collect = [&](int step, float (&out)[EPT]) -> int {
    int fail = 0;
    const unsigned long long* pbuf = gpart + (size_t)(step & 1) * psz;
    const unsigned long long* src[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const int n = qq * U + (eu[e] - u0);
      src[e] = pbuf + ((size_t)(pg * 4) * Bp + (ev[e] ? eb[e] : 0)) * UG + (ev[e] ? n : 0);
    }
    unsigned long long v[EPT][4];
    Spin sp(p.wait_ticks);
    for (;;) {
#pragma unroll
      for (int e = 0; e < EPT; ++e)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          v[e][k] = 0ull;
          if (ev[e] && k < nq) v[e][k] = __hip_atomic_load(src[e] + (size_t)k * Bp * UG, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      bool ok = true;
#pragma unroll
      for (int e = 0; e < EPT; ++e)
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (ev[e] && k < nq) ok = ok && (unsigned)(v[e][k] >> 32) == (unsigned)(step + 1);
      if (ok) break;
      if (sp.expired(p.err)) { fail = 1; break; }
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      float sum = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) sum += __uint_as_float((unsigned)v[e][k]);
      out[e] = ev[e] ? sum : 0.f;
    }
    return fail;
  };

  // Step s sums the partial tiles of step s-1, also when step s-1 was the last step of the
  // previous launch: flags, exchange arrays and tagged tiles live in device memory.
  for (int s = s_begin; s < s_end; ++s) {
    const int t = frame_of(s);
    char* dzcur = dzbase + (size_t)(s & 1) * xsz;
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
      test_delay(p.slow_wg, p.slow_ticks);
      const float* in = bin + (s & 1) * 7 * NE;
      float* out = dzo + (s & 1) * 4 * NE;
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        vprev[e] = false;
        if (!ev[e]) continue;
        const int j = tid + e * 256;
        float dz[4] = {0.f, 0.f, 0.f, 0.f};
        const bool m = t < elen[e];
        vprev[e] = m;
        if (m) {
          const float gi = in[0 * NE + j], gf = in[1 * NE + j], go = in[2 * NE + j], gg = in[3 * NE + j];
          const float tc = ftanh(in[4 * NE + j]);
          const float dh = in[6 * NE + j] + Dh[e];
          const float d_o = dh * tc;
          const float dc = Dc[e] + dh * go * (1.0f - tc * tc);
          dz[0] = dc * gg * gi * (1.0f - gi);
          dz[1] = dc * in[5 * NE + j] * gf * (1.0f - gf);
          dz[2] = d_o * go * (1.0f - go);
          dz[3] = dc * gi * (1.0f - gg * gg);
          Dc[e] = dc * gf;
        }
        if (BF) {
          // the 4 gates of a unit are 4 consecutive k: one 8-byte word of bf16
          const unsigned long long w = (unsigned long long)bf16_bits(dz[0]) | ((unsigned long long)bf16_bits(dz[1]) << 16) |
                                       ((unsigned long long)bf16_bits(dz[2]) << 32) | ((unsigned long long)bf16_bits(dz[3]) << 48);
          __hip_atomic_store(reinterpret_cast<unsigned long long*>(dzcur) + (eslot[e] >> 2), w, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        }
        if (P3) {
          // the same 8-byte word of four gates, once per part (a part's chunks are nchp * 1024 bytes on)
          unsigned long long w1 = 0ull, w2 = 0ull, w3 = 0ull;
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            unsigned b1, b2, b3;
            cut3_bits(dz[g], b1, b2, b3);
            w1 |= (unsigned long long)b1 << (16 * g); w2 |= (unsigned long long)b2 << (16 * g); w3 |= (unsigned long long)b3 << (16 * g);
          }
          unsigned long long* dst = reinterpret_cast<unsigned long long*>(dzcur) + (eslot[e] >> 2);
          __hip_atomic_store(dst, w1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(dst + nchp * 128, w2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(dst + 2 * nchp * 128, w3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          // fp32: rows (unit, gate 0..3) are 16 lanes apart in operand order
          if (!BF && !P3) st_dev(reinterpret_cast<float*>(dzcur) + eslot[e] + g * 64, dz[g]);
          out[g * NE + j] = dz[g];
          dbacc[e][g] += dz[g];
        }
      }
      wait_stores_acked();
    } else {
      // stage the next frame's inputs (loaded a step ago), write out the previous frame's d a,
      // start loading the frame after next: every wait here is on work issued a step ago
      if (s + 1 < s_end) io_stage(s + 1);
      if (s > s_begin) io_store(s - 1);
      if (s + 2 < s_end) io_load(s + 2);
    }
    if (barrier_any_failed(fail, failed)) {
      if (tid == 0) st_dev(p.err, 1u);
      return;
    }
    if ((int)blockIdx.x != p.mute_wg) publish_flag(gflags, wg, (unsigned)(s + 1));

    // this workgroup's quarter of d a_t R^T for its unit group
    fail = 0;
    if (!is_io && qq < nq) {
      if (!wave_wait_flags(myflags, prod_first, prod_count, Gb, (unsigned)(s + 1), p.err, p.wait_ticks)) fail = 1;
      floatx4 acc[MT][NT];
      if (P3) wave_product_3<MT, NT>(dzcur + (size_t)(qq * 4 + wave) * wbytes, wbytes, nchp, RTb + (size_t)wave * Hq * UG, 4 * Hq * UG, acc);
      else if (BF) wave_product_bf<MT, NT, HALF, true>(dzcur + (size_t)(qq * 4 + wave) * wbytes, wbytes, nch, RTb + (size_t)wave * Hq * UG, acc);
      else wave_product<MT, NT, HALF>(reinterpret_cast<const float*>(dzcur + (size_t)(qq * 4 + wave) * wbytes), wbytes, nch,
                                      RTs + (size_t)wave * Hq * UG, acc);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          *reinterpret_cast<floatx4*>(Red + ((wave * MT + mt) * NT + nt) * 256 + lane * 4) = acc[mt][nt];
    }
    if (barrier_any_failed(fail, failed + 1)) {
      if (tid == 0) st_dev(p.err, 1u);
      return;
    }
    // sum the four wavefronts' tiles in order and hand (value, tag) to the owners
    if (!is_io && qq < nq) {
      unsigned long long* pbuf = gpart + (size_t)(s & 1) * psz + (size_t)(pg * 4 + qq) * Bp * UG;
      const int ln = tid >> 2, reg = tid & 3;
      const int row = 4 * (ln >> 4) + reg, col = ln & 15;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          if (HALF && row >= 8) continue;          // rows that hold no sequence: nobody reads them
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
    io_store(s_end - 1);
  } else if (s_end == T) {
    float g[EPT];
    fail = collect(T - 1, g);
#pragma unroll
    for (int e = 0; e < EPT; ++e) Dh[e] = vprev[e] ? g[e] : g[e] + Dh[e];
  }
  if (barrier_any_failed(fail, failed)) {
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
    const size_t bu = (size_t)(b0 + eb[e]) * H + eu[e];
    if (s_end < T) { D.dhstate[bu] = Dh[e]; D.dcstate[bu] = Dc[e]; }
    else {
      if (D.dh0) D.dh0[bu] = Dh[e];
      if (D.dc0) D.dc0[bu] = Dc[e];
    }
  }
  __syncthreads();
  if (tid < 4 * U) {
    const int g = tid / U, u = u0 + tid % U;
    if (u < H) {
      // launches that split the T steps add their share in launch order; with several groups of
      // sequences each group keeps its own sum (added up in group order by a kernel that follows)
      float sum = 0.f;
      for (int b = 0; b < B; ++b) sum += stage[b * 4 * U + tid];
      float* dst = (p.NG > p.ndir ? D.dbpart + (size_t)bgi * 4 * H : D.db) + g * H + u;
      *dst = s_begin > 0 ? *dst + sum : sum;
    }
  }
}

// ---------------------------------------------------------------------------
// backward, one exchange per step (groups of at most 16 sequences, fp32)
// ---------------------------------------------------------------------------
// The kernel above needs two exchanges per step (d a_t to the multipliers, partial tiles back to the owners), and
// an exchange between CUs costs 2.7 us whatever its size up to a few tens of KB.  Here the sum over k of
// d h_{t-1}[b, j] = sum_k d a_t[b, k] R[j, k] is split by the OWNERS of k instead: the workgroup that owns U units
// multiplies its own d a_t[16 x 4U] (never leaves the CU) with its [4U x Hp] rows of R^T (the slice the forward
// kernel keeps, transposed) and hands every other workgroup c the [16 x U] piece that belongs to c's units; the
// owners add the pieces of all producers in a fixed order.  One exchange per step; in return every workgroup
// writes 16 x Hp floats per step (32 KiB at H = 500) instead of 2 + 4 KiB and reads as much (bare exchange at
// 4 groups of 64 workgroups: 3.4 us against 2.75 + 2.8 us for the two hops).
//
// Exchange array of a group: [step parity][consumer c][producer w][q = 4][n = U][i = 4] floats, element
// (sequence 4q + i, unit c*U + n): a lane's four accumulator values of an MFMA tile (rows 4q..4q+3 of one column)
// are one 16-byte store, and a consumer's pieces of all producers are contiguous.
struct PBwd1Params {
  PBwdDir d[2];
  float* px[kMaxGroups];           // per group: 2 x [Gm][Gm][16 U] floats
  unsigned* flags[kMaxGroups];     // per group: [flag copies][Gm]
  int ndir, NG, Bg;
  const int32_t* seq_lens;
  unsigned* err;
  unsigned long long wait_ticks;
  int mute_wg;
  int slow_wg; unsigned slow_ticks;
  int T, B, H, ldy, Gm;
  int s_begin, s_end;
};

// NT: U = 4 NT units per workgroup; TN: the product's 64 TN columns (>= H) are dealt out to the 4 wavefronts, TN
// MFMA column tiles each.
template <int NT, int TN>
__global__ __launch_bounds__(kBlockThreads) void lstm_bwd_onehop_kernel(PBwd1Params p) {
  constexpr int U = 4 * NT, KZ = 16 * NT;        // units; rows of the resident slice = (gate, unit) pairs
  constexpr int HP = 64 * TN;                    // columns of the resident slice (units of the layer, padded)
  constexpr int NE = 16 * U;                     // (sequence, unit) pairs owned by this workgroup
  constexpr int EPL = NE / 64;                   // pairs per I/O lane
  constexpr int VEC = 4 * U;                     // 16-byte vectors of one producer's piece
  constexpr int SUB = 64 / VEC;                  // producers a wavefront loads side by side (VEC <= 64)
  constexpr int LD = U;                          // loads per lane: 16 producers per wavefront / SUB
  constexpr int NPART = 4 * SUB;                 // partial sums per vector
  static_assert(VEC <= 64 && 16 % SUB == 0, "piece must fit a wavefront");
  extern __shared__ __align__(16) float lds[];
  const int grp = blockIdx.x % p.NG, wg = blockIdx.x / p.NG;
  const int dir = grp % p.ndir, bgi = grp / p.ndir, b0 = bgi * p.Bg;
  const PBwdDir& D = p.d[dir];
  const int T = p.T, H = p.H, Gm = p.Gm;
  const int B = min(p.Bg, p.B - b0);
  if (B <= 0) return;
  const int s_begin = p.s_begin, s_end = p.s_end;
  if (ld_dev(p.err) != 0u) return;               // an earlier launch of this pass gave up waiting
  __builtin_amdgcn_s_setprio(3);
  const int u0 = wg * U;
  float* RTs = lds;                              // [KZ][HP], columns rotated per row
  float* Red = RTs + (size_t)KZ * HP;            // [NPART][VEC][4] partial sums of the pieces
  float* Az = Red + NPART * VEC * 4;             // [KZ][16]   d a of the frame, MFMA operand order
  float* bin = Az + KZ * 16;                     // [2][7][NE] gates i,f,o,g, c, c_prev, dy of the frame
  float* dzo = bin + 2 * 7 * NE;                 // [2][4][NE] d a of the frame (for the I/O wavefront)
  int* failed = reinterpret_cast<int*>(dzo + 2 * 4 * NE);

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool is_io = wave == 4;
  const int lane = tid & 63;

  // resident slice: row k = g*U + uu (gate g of owned unit uu), column j (unit of the layer):  R[j][g*H + u0 + uu]
  for (int idx = tid; idx < KZ * HP; idx += kBlockThreads) {
    const int k = idx / HP, j = idx % HP;
    const int g = k / U, u = u0 + k % U;
    const float v = (j < H && u < H) ? D.R[(size_t)j * 4 * H + g * H + u] : 0.f;
    RTs[k * HP + ((j + 16 * (k & 3)) & (HP - 1))] = v;
  }

  const size_t piece = (size_t)16 * U;                         // floats of one (consumer, producer) piece
  const size_t pxsz = (size_t)Gm * Gm * piece;                 // floats of one step buffer
  float* const pxbase = p.px[grp];
  unsigned* const gflags = p.flags[grp];

  // the pair (sequence, unit) a compute thread owns (threads NE.. of the compute wavefronts own none)
  const int eb = tid / U, eu = u0 + tid % U;
  const bool ev = !is_io && tid < NE && eb < B && eu < H;
  float Dh = 0.f, Dc = 0.f, dbacc[4] = {0.f, 0.f, 0.f, 0.f};
  int elen = 0;
  bool vprev = false;
  if (ev) {
    const size_t bu = (size_t)(b0 + eb) * H + eu;
    elen = min(max(p.seq_lens[b0 + eb], 0), T);
    if (s_begin > 0) {
      Dh = D.dhstate[bu]; Dc = D.dcstate[bu];
      const int tlast = D.direction > 0 ? T - s_begin : s_begin - 1;   // frame of step s_begin - 1
      vprev = tlast < elen;
    } else {
      if (D.dhT) Dh = D.dhT[bu];
      if (D.dcT) Dc = D.dcT[bu];
    }
  }

  // I/O lanes (as in the kernel above)
  int ib[EPL], iu[EPL];
  bool iv[EPL];
  float lr[EPL][6];
  float cnext[EPL];
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
    const int tprev = D.direction > 0 ? t - 1 : t + 1;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      if (!iv[i]) continue;
      const size_t row = (size_t)t * p.B + b0 + ib[i];
      const float* zrow = D.zg + row * 4 * H + iu[i];
      lr[i][0] = zrow[0]; lr[i][1] = zrow[H]; lr[i][2] = zrow[2 * H]; lr[i][3] = zrow[3 * H];
      if (tprev >= 0 && tprev < T) lr[i][4] = D.c[((size_t)tprev * p.B + b0 + ib[i]) * H + iu[i]];
      else lr[i][4] = D.c0 ? D.c0[(size_t)(b0 + ib[i]) * H + iu[i]] : 0.f;
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
      float* zrow = D.zg + ((size_t)t * p.B + b0 + ib[i]) * 4 * H + iu[i];
      zrow[0] = src[0 * NE + j]; zrow[H] = src[1 * NE + j]; zrow[2 * H] = src[2 * NE + j]; zrow[3 * H] = src[3 * NE + j];
    }
  };
  if (is_io) {
    const int t0 = frame_of(s_begin);
#pragma unroll
    for (int i = 0; i < EPL; ++i)
      if (iv[i]) cnext[i] = D.c[((size_t)t0 * p.B + b0 + ib[i]) * H + iu[i]];
    io_load(s_begin);
    io_stage(s_begin);
    if (s_begin + 1 < s_end) io_load(s_begin + 1);
  }
  if (tid < 2) failed[tid] = 0;
  __syncthreads();

  // wavefront `wave` takes the pieces of producers [16 wave, 16 wave + 16): lane = (sub, vector)
  const int sub = lane / VEC, vec = lane % VEC;
  const unsigned* myflags = gflags + (wg % kFlagCopies) * kFlagCopyStride;

  // pieces of step `step` for this workgroup's units -> Red[NPART][VEC] (each a fixed-order sum over LD producers)
  auto collect = [&](int step) -> int {
    int fail = 0;
    if (!wave_wait_flags(myflags, wave * 16, 16, Gm, (unsigned)(step + 1), p.err, p.wait_ticks)) fail = 1;
    const float* mine = pxbase + (size_t)(step & 1) * pxsz + (size_t)wg * Gm * piece;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(mine), 0, (int)(Gm * piece * 4), 0x00020000);
    floatx4 v[LD];
#pragma unroll
    for (int k = 0; k < LD; ++k) {
      const int w = wave * 16 + k * SUB + sub;                  // producers past Gm read beyond the resource: zeros
      v[k] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)((w * piece + vec * 4) * 4), 0, kAuxSc1));
    }
    floatx4 sum = v[0];
#pragma unroll
    for (int k = 1; k < LD; ++k) sum += v[k];
    *reinterpret_cast<floatx4*>(Red + ((wave * SUB + sub) * VEC + vec) * 4) = sum;
    return fail;
  };
  // the owned pair's sum over the NPART partial sums, in order
  auto gathered = [&]() -> float {
    const int v = (eb >> 2) * U + (eu - u0), i = eb & 3;
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < NPART; ++k) sum += Red[(k * VEC + v) * 4 + i];
    return sum;
  };

  for (int s = s_begin; s < s_end; ++s) {
    const int t = frame_of(s);
    int fail = 0;
    if (!is_io) {
      if (s > 0) fail = collect(s - 1);
    } else {
      if (s + 1 < s_end) io_stage(s + 1);
      if (s > s_begin) io_store(s - 1);
      if (s + 2 < s_end) io_load(s + 2);
    }
    if (barrier_any_failed(fail, failed)) {
      if (tid == 0) st_dev(p.err, 1u);
      return;
    }
    test_delay(p.slow_wg, p.slow_ticks);
    // gate derivatives of the owned pairs; d a of the frame in MFMA operand order and for the I/O wavefront
    if (!is_io && tid < NE) {
      float dz[4] = {0.f, 0.f, 0.f, 0.f};
      if (ev) {
        if (s > 0) { const float g = gathered(); Dh = vprev ? g : g + Dh; }
        const float* in = bin + (s & 1) * 7 * NE;
        const bool m = t < elen;
        vprev = m;
        if (m) {
          const float gi = in[0 * NE + tid], gf = in[1 * NE + tid], go = in[2 * NE + tid], gg = in[3 * NE + tid];
          const float tc = ftanh(in[4 * NE + tid]);
          const float dh = in[6 * NE + tid] + Dh;
          const float d_o = dh * tc;
          const float dc = Dc + dh * go * (1.0f - tc * tc);
          dz[0] = dc * gg * gi * (1.0f - gi);
          dz[1] = dc * in[5 * NE + tid] * gf * (1.0f - gf);
          dz[2] = d_o * go * (1.0f - go);
          dz[3] = dc * gi * (1.0f - gg * gg);
          Dc = dc * gf;
        }
      }
      float* out = dzo + (s & 1) * 4 * NE;
      const int uu = tid % U;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        Az[(g * U + uu) * 16 + eb] = dz[g];
        out[g * NE + tid] = dz[g];
        dbacc[g] += dz[g];
      }
    }
    __syncthreads();
    // this workgroup's d a_t times its rows of R^T: the wavefront's 16 TN columns of the [16 x HP] result
    if (!is_io) {
      const int l16 = lane & 15, lq = lane >> 4;
      floatx4 acc[TN];
#pragma unroll
      for (int nt = 0; nt < TN; ++nt) acc[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
      // the rotation of a row's columns, 16 (k % 4) = 16 lq, is the same for every row this lane reads: one LDS
      // address per column tile, and k-step ks at a constant distance 4 ks HP from k-step 0
      const float* brow[TN];
#pragma unroll
      for (int nt = 0; nt < TN; ++nt)
        brow[nt] = RTs + (size_t)lq * HP + (((wave * TN + nt) * 16 + l16 + 16 * lq) & (HP - 1));
      // operands of k-step ks + 1 are fetched from LDS while the MFMAs of k-step ks run; the scheduling barriers keep
      // the compiler from fetching all k-steps at once (which costs 50 registers more and, beside the matrix-product
      // kernels that share the CU, one of their two workgroups)
      float a_cur = Az[lq * 16 + l16], b_cur[TN];
#pragma unroll
      for (int nt = 0; nt < TN; ++nt) b_cur[nt] = brow[nt][0];
#pragma unroll
      for (int ks = 0; ks < KZ / 4; ++ks) {
        float a_next = 0.f, b_next[TN];
        if (ks + 1 < KZ / 4) {
          a_next = Az[((ks + 1) * 4 + lq) * 16 + l16];
#pragma unroll
          for (int nt = 0; nt < TN; ++nt) b_next[nt] = brow[nt][(size_t)(ks + 1) * 4 * HP];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur, b_cur[nt], acc[nt], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (ks + 1 < KZ / 4) {
          a_cur = a_next;
#pragma unroll
          for (int nt = 0; nt < TN; ++nt) b_cur[nt] = b_next[nt];
        }
      }
      // lane (lq, l16) of tile nt holds rows 4 lq .. 4 lq + 3 of column j: one 16-byte store into the piece of j's owner
      float* cur = pxbase + (size_t)(s & 1) * pxsz;
      __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(cur, 0, (int)(pxsz * 4), 0x00020000);
#pragma unroll
      for (int nt = 0; nt < TN; ++nt) {
        const int j = (wave * TN + nt) * 16 + l16;
        const int c = j / U, n = j % U;
        if (c < Gm) {
          const size_t off = ((size_t)c * Gm + wg) * piece + (size_t)(lq * U + n) * 4;
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(intx4, acc[nt]), wr, (int)(off * 4), 0, kAuxSc1);
        }
      }
      wait_stores_acked();
    }
    __syncthreads();
    if ((int)blockIdx.x != p.mute_wg) publish_flag(gflags, wg, (unsigned)(s + 1));
  }

  int fail = 0;
  if (is_io) {
    io_store(s_end - 1);
  } else if (s_end == T) {
    fail = collect(T - 1);
  }
  if (barrier_any_failed(fail, failed + 1)) {
    if (tid == 0) st_dev(p.err, 1u);
    return;
  }
  if (ev && s_end == T) { const float g = gathered(); Dh = vprev ? g : g + Dh; }
  __syncthreads();                               // Red is reused as the bias gradient's stage below
  float* stage = Red;                            // [16][4U]
  if (!is_io && tid < NE) {
    const int uu = tid % U;
#pragma unroll
    for (int g = 0; g < 4; ++g) stage[eb * 4 * U + g * U + uu] = ev ? dbacc[g] : 0.f;
    if (ev) {
      const size_t bu = (size_t)(b0 + eb) * H + eu;
      if (s_end < T) { D.dhstate[bu] = Dh; D.dcstate[bu] = Dc; }
      else {
        if (D.dh0) D.dh0[bu] = Dh;
        if (D.dc0) D.dc0[bu] = Dc;
      }
    }
  }
  __syncthreads();
  if (tid < 4 * U) {
    const int g = tid / U, u = u0 + tid % U;
    if (u < H) {
      float sum = 0.f;
      for (int b = 0; b < B; ++b) sum += stage[b * 4 * U + tid];
      float* dst = (p.NG > p.ndir ? D.dbpart + (size_t)bgi * 4 * H : D.db) + g * H + u;
      *dst = s_begin > 0 ? *dst + sum : sum;
    }
  }
}

// ---------------------------------------------------------------------------
// set-up kernels: clear flags, exchange arrays and tags; seed h0 in operand order;
// add up the bias gradients of the groups of sequences
// ---------------------------------------------------------------------------
struct PrepParams {
  unsigned* zero_words; size_t nzero;             // flags + exchange (+ partial tiles) of all groups
  void* hx1[kMaxGroups]; const float* h0[2];      // forward only: buffer 1 of each group's h exchange, h0 or null
  int ndir, B, Bg, H, KW, wbytes, MT, prec;   // prec: 0 fp32, 1 bf16, 2 three bf16 parts (see the kernels)
};
__global__ __launch_bounds__(256) void prep_kernel(PrepParams p) {
  const size_t gtid = (size_t)blockIdx.x * 256 + threadIdx.x, gsz = (size_t)gridDim.x * 256;
  for (size_t i = gtid; i < p.nzero; i += gsz) p.zero_words[i] = 0u;
}
// runs after prep_kernel (same stream): h0 lands in words that kernel has cleared
__global__ __launch_bounds__(256) void seed_h0_kernel(PrepParams p) {
  const size_t gtid = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (gtid >= (size_t)p.B * p.H) return;
  const int bglob = (int)(gtid / p.H), u = (int)(gtid % p.H);
  const int bgi = bglob / p.Bg, b = bglob % p.Bg;      // group of sequences, index inside it
  for (int d = 0; d < p.ndir; ++d) {
    if (!p.h0[d]) continue;
    void* hx1 = p.hx1[bgi * p.ndir + d];
    const int k = u % p.KW;
    int slot;
    if (p.prec != 0) {
      if (p.MT == 1) slot = operand_slot_bf<1>(k, b);
      else if (p.MT == 2) slot = operand_slot_bf<2>(k, b);
      else if (p.MT == 3) slot = operand_slot_bf<3>(k, b);
      else slot = operand_slot_bf<4>(k, b);
      unsigned short* dst = static_cast<unsigned short*>(hx1) + (size_t)(u / p.KW) * (p.wbytes / 2) + slot;
      if (p.prec == 1) *dst = bf16_bits(p.h0[d][gtid]);
      else {
        unsigned b1, b2, b3;
        cut3_bits(p.h0[d][gtid], b1, b2, b3);
        const size_t part = (size_t)(p.wbytes / 3) / 2;        // bf16 elements of one part of a wavefront's block
        dst[0] = (unsigned short)b1; dst[part] = (unsigned short)b2; dst[2 * part] = (unsigned short)b3;
      }
    } else {
      if (p.MT == 1) slot = operand_slot<1>(k, b);
      else if (p.MT == 2) slot = operand_slot<2>(k, b);
      else if (p.MT == 3) slot = operand_slot<3>(k, b);
      else slot = operand_slot<4>(k, b);
      static_cast<float*>(hx1)[(size_t)(u / p.KW) * (p.wbytes / 4) + slot] = p.h0[d][gtid];
    }
  }
}
struct DbSumParams { float* db[2]; const float* dbpart[2]; int ndir, nb, n; };
__global__ __launch_bounds__(256) void db_sum_kernel(DbSumParams p) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= p.n) return;
  for (int d = 0; d < p.ndir; ++d) {
    float sum = 0.f;
    for (int g = 0; g < p.nb; ++g) sum += p.dbpart[d][(size_t)g * p.n + i];
    p.db[d][i] = sum;
  }
}

// ---- host side ----------------------------------------------------------------
unsigned long long g_wait_ticks = kDefaultWaitTicks;
int g_mute_wg = -1;
int g_slow_wg = -1;
unsigned g_slow_ticks = 0;
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
constexpr size_t kFlagBytes = (size_t)kFlagCopies * kFlagCopyStride * sizeof(unsigned);

struct Plan {
  bool ok;
  int ROWS, MT, NT, U, UG, Bp, prec;
  int nb, Bg, NG;                                // groups of sequences per direction, sequences per group, all groups
  int Gf, Hp, nchF;
  int PG, Gb, Hq, nchB;
  size_t ldsF, ldsB;
  bool onehop;                                   // backward pass with one exchange per step (lstm_bwd_onehop_kernel)
  int TN;                                        // its column tiles per wavefront (64 TN >= H)
  size_t ldsB1, px_bytes;                        // its LDS request; bytes of its exchange array per group
};

// kernels exist for these (ROWS, NT)
inline bool have_kernel(int rows, int nt) {
  if (nt == 1) return rows >= 16;
  if (nt == 2) return true;
  return rows <= 16;                             // nt == 4
}

// One plan for a given number nb of groups of sequences per direction, or !ok.
Plan plan_for(const RecShape& s, int num_cus, size_t max_lds, int nb) {
  Plan pl{};
  pl.ok = false;
  const int bf = s.operand_dtype == 1 ? 1 : 0;
  const int NG = s.ndir * nb;
  if (NG > kMaxGroups || nb > s.B) return pl;
  const int Bg = (s.B + nb - 1) / nb;
  if (Bg > 64) return pl;
  const int per_group = num_cus / NG;
  // the backward kernel with one exchange per step needs at most 64 workgroups per group: when it is asked for, the
  // first round only takes slice widths that allow it
  for (int round = (s.bwd_exchange == 2 && !bf && Bg <= 16 && s.H <= 512) ? 0 : 1; round < 2; ++round)
  for (int NT = 1; NT <= 4; NT *= 2) {
    if (round == 0 && (s.H + 4 * NT - 1) / (4 * NT) > 64) continue;
    const int rows = Bg <= 8 && have_kernel(8, NT) ? 8 : (Bg <= 16 ? 16 : (Bg <= 32 ? 32 : (Bg <= 48 && have_kernel(48, NT) ? 48 : 64)));
    if (!have_kernel(rows, NT)) continue;
    const int MT = rows <= 16 ? 1 : rows / 16;
    const int U = 4 * NT, UG = 16 * NT;
    const int Gf = (s.H + U - 1) / U;
    const int PG = (s.H + UG - 1) / UG;
    const int Gb = 4 * PG;
    if (Gf > per_group || Gb > per_group) continue;
    const int Hq = (int)align_up((size_t)PG * U, 32);
    const size_t red = (size_t)4 * MT * NT * 256;
    const size_t ne = (size_t)rows * U;
    // fp32 operands with two or more 16-row tiles per workgroup: the three-part kernels where their 1.5 x larger
    // resident matrix fits (at most 4 k-steps per wavefront: 512 units), else the fp32 matrix instructions
    int prec = bf;
    int Hp = (int)align_up((size_t)s.H, bf ? 128 : 64);          // rows of h per wavefront: whole MFMA k-steps
    size_t es = bf ? 2 : 4;                      // bytes per element of the resident matrix and the exchanged rows
    if (!bf && !s.fp32_instructions && MT >= 2 && s.H <= 512) {
      const int Hp3 = (int)align_up((size_t)s.H, 128);
      const size_t lf3 = (size_t)Hp3 * 16 * NT * 6 + (red + (2 * 4 + 2 * 6) * ne) * sizeof(float) + 16;
      const size_t lb3 = (size_t)4 * Hq * UG * 6 + (red + (2 * 7 + 2 * 4) * ne) * sizeof(float) + 16;
      if (lf3 <= max_lds && lb3 <= max_lds && Hq % 32 == 0) { prec = 2; Hp = Hp3; es = 6; }
    }
    // a wavefront polls at most 64 producers
    if (Hp / 4 / U > 64 || Hq / 4 / U > 64) continue;
    const size_t lf = (size_t)Hp * 16 * NT * es + (red + (2 * 4 + 2 * 6) * ne) * sizeof(float) + 16;
    const size_t lb = (size_t)4 * Hq * UG * es + (red + (2 * 7 + 2 * 4) * ne) * sizeof(float) + 16;
    if (lf > max_lds || lb > max_lds) continue;
    // One workgroup per CU: request more than half of the CU's LDS so that the dispatcher cannot
    // stack two of these workgroups on one CU (they would share its matrix cores and every other
    // workgroup would wait for them each step).
    const size_t exclusive = max_lds / 2 + 1024;
    pl.ok = true; pl.ROWS = rows; pl.MT = MT; pl.NT = NT; pl.U = U; pl.UG = UG; pl.Bp = 16 * MT; pl.prec = prec;
    pl.nb = nb; pl.Bg = Bg; pl.NG = NG;
    // 16-byte chunks per lane and wavefront: fp32 4 values (4 k-steps x batch tiles / 4), bf16 8 values (1 k-step of 32)
    // (three parts: the chunks of all three)
    pl.Gf = Gf; pl.Hp = Hp; pl.nchF = prec ? (prec == 2 ? 3 : 1) * (Hp / 4 / 32) * MT : (Hp / 16) * MT / 4;
    pl.PG = PG; pl.Gb = Gb; pl.Hq = Hq; pl.nchB = prec ? (prec == 2 ? 3 : 1) * (Hq / 32) * MT : (Hq / 4) * MT / 4;
    pl.ldsF = lf > exclusive ? lf : exclusive; pl.ldsB = lb > exclusive ? lb : exclusive;
    // One exchange per step in the backward pass: groups of at most 16 sequences (one MFMA row tile), fp32, the
    // forward kernel's deal of the units (Gf <= 64 workgroups), at most 512 units.
    pl.onehop = false; pl.TN = 0; pl.ldsB1 = 0; pl.px_bytes = 0;
    if (!bf && rows <= 16 && Gf <= 64 && s.H <= 512 && s.bwd_exchange == 2) {
      int TN = 1;
      while (64 * TN < s.H) TN *= 2;
      const size_t l1 = ((size_t)16 * NT * 64 * TN + 1024 + (size_t)16 * NT * 16 + (2 * 7 + 2 * 4) * 16 * U) * sizeof(float) + 16;
      if (l1 <= max_lds) {
        pl.onehop = true; pl.TN = TN;
        pl.ldsB1 = l1 > exclusive ? l1 : exclusive;
        pl.px_bytes = align_up((size_t)2 * Gf * Gf * 16 * U * sizeof(float), 256);
      }
    }
    return pl;
  }
  return pl;
}

// The sequences of a minibatch are independent, so they can be dealt out to nb groups of
// workgroups per direction, each group holding its own copy of the recurrent matrix (spread over
// fewer, larger slices) and exchanging h_t / d a_t only among its own members.  Smaller groups
// exchange faster (fewer producers to wait for, fewer bytes per consumer); in return each
// workgroup multiplies a larger slice, and below 16 sequences per group the 16-row MFMA tiles
// are partly empty.  Preferred: the largest nb that leaves at least 16 sequences per group.
Plan make_plan(const RecShape& s, int num_cus, size_t max_lds) {
  Plan none{};
  none.ok = false;
  if (s.operand_dtype != 0 && s.operand_dtype != 1) return none;
  if (s.B < 1 || s.H < 1 || s.ndir < 1 || s.ndir > 2) return none;
  if (s.batch_groups > 0) return plan_for(s, num_cus, max_lds, s.batch_groups);
  int first = 1;
  while (first * 2 * s.ndir <= kMaxGroups && (s.B + first * 2 - 1) / (first * 2) >= 16) first *= 2;
  for (int nb = first; nb >= 1; nb /= 2) {
    const Plan pl = plan_for(s, num_cus, max_lds, nb);
    if (pl.ok) return pl;
  }
  for (int nb = first * 2; nb * s.ndir <= kMaxGroups; nb *= 2) {   // more sequences than one group can hold
    const Plan pl = plan_for(s, num_cus, max_lds, nb);
    if (pl.ok) return pl;
  }
  return none;
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

// Scratch layout (bytes), independent of the device: per group [flag copies][exchange arrays]
// [partial tiles], then per direction [2 state arrays][per-group bias gradients].  Sized for the
// worst case over the numbers of groups a plan may choose.
struct GroupBytes { size_t exch, part, total; };
GroupBytes group_bytes(const RecShape& s, int nb) {
  const size_t Bg = ((size_t)s.B + nb - 1) / nb;
  const size_t Bp = Bg <= 16 ? 16 : (Bg <= 32 ? 32 : 64);
  const size_t Hp = align_up((size_t)s.H, 128);
  const size_t Hq = align_up((size_t)s.H / 4 + 16, 32);
  GroupBytes g;
  // 4 bytes per exchanged value; 6 where fp32 operands may be exchanged as three bf16 parts
  g.exch = align_up(2 * (Hp > 16 * Hq ? Hp : 16 * Hq) * Bp * (s.operand_dtype == 0 ? 6 : 4), 256);
  g.part = align_up(2 * 4 * Bp * ((size_t)s.H + 64) * sizeof(unsigned long long), 256);
  g.total = kFlagBytes + g.exch + g.part;
  return g;
}
size_t groups_bytes_max(const RecShape& s) {
  size_t m = 0;
  for (int nb = 1; nb * s.ndir <= kMaxGroups; nb *= 2) {
    const size_t v = (size_t)nb * s.ndir * group_bytes(s, nb).total;
    if (v > m) m = v;
  }
  return m;
}
// Upper bound of the one-exchange backward kernel's arrays over all plans a device may get (they sit behind the
// other scratch and are not needed by the forward pass): NG groups of 2 x Gm x Gm pieces of 16 U floats, Gm = ceil(H / U).
size_t onehop_bytes_max(const RecShape& s) {
  if (s.operand_dtype != 0 || s.H > 512) return 0;
  size_t m = 0;
  for (int nb = 1; nb * s.ndir <= kMaxGroups; nb *= 2) {
    if (((size_t)s.B + nb - 1) / nb > 16) continue;
    for (int U = 4; U <= 16; U *= 2) {
      const size_t Gm = ((size_t)s.H + U - 1) / U;
      if (Gm > 64) continue;
      const size_t v = (size_t)nb * s.ndir * align_up(2 * Gm * Gm * 16 * U * sizeof(float), 256);
      if (v > m) m = v;
    }
  }
  return m;
}
size_t state_bytes(const RecShape& s) { return align_up((size_t)s.B * s.H * sizeof(float), 256); }
size_t dbpart_bytes(const RecShape& s) { return align_up((size_t)kMaxGroups * 4 * s.H * sizeof(float), 256); }
// per-direction arrays behind the groups: which = 0, 1 state arrays, 2 per-group bias gradients
float* dir_array(char* scratch, const RecShape& s, int d, int which) {
  char* base = scratch + groups_bytes_max(s) + (size_t)d * (2 * state_bytes(s) + dbpart_bytes(s));
  return reinterpret_cast<float*>(base + (size_t)which * state_bytes(s));
}

}  // namespace

void persistent_test_hook(int mute_workgroup, unsigned long long wait_ticks) {
  g_mute_wg = mute_workgroup;
  g_wait_ticks = wait_ticks ? wait_ticks : kDefaultWaitTicks;
}

void persistent_test_delay(int slow_workgroup, unsigned ticks) {
  g_slow_wg = slow_workgroup;
  g_slow_ticks = slow_workgroup >= 0 ? ticks : 0u;
}

bool persistent_supported(const RecShape& s, int num_cus, size_t max_lds) {
  return make_plan(s, num_cus, max_lds).ok;
}

size_t persistent_lds_bytes(const RecShape& s, int num_cus, size_t max_lds) {
  const Plan pl = make_plan(s, num_cus, max_lds);
  if (!pl.ok) return 0;
  const size_t b = pl.onehop ? pl.ldsB1 : pl.ldsB;
  return pl.ldsF > b ? pl.ldsF : b;
}

bool persistent_plan_info(const RecShape& s, int num_cus, size_t max_lds, int out[10]) {
  const Plan pl = make_plan(s, num_cus, max_lds);
  if (!pl.ok) return false;
  out[0] = pl.NG; out[1] = pl.Bg; out[2] = pl.ROWS; out[3] = pl.U;
  out[4] = pl.Gf; out[5] = pl.onehop ? pl.Gf : pl.Gb; out[6] = pl.Hp; out[7] = pl.onehop ? 64 * pl.TN : pl.Hq;
  out[8] = pl.onehop ? 1 : 2; out[9] = pl.prec;
  return true;
}

namespace {
// the kernel of a plan's precision; the three-part kernels exist for two and more 16-row tiles only
template <int ROWS, int NT>
hipError_t launch_fwd_prec(int prec, int grid, size_t lds, int num_cus, hipStream_t stream, void* kp, int* resident_err) {
  if (prec == 1) return resident_launch(lstm_fwd_persistent_kernel<ROWS, NT, 1>, grid, kBlockThreads, lds, num_cus, stream, kp, resident_err);
  if constexpr (ROWS >= 32) {
    if (prec == 2) return resident_launch(lstm_fwd_persistent_kernel<ROWS, NT, 2>, grid, kBlockThreads, lds, num_cus, stream, kp, resident_err);
  }
  if (prec != 0) return hipErrorInvalidValue;
  return resident_launch(lstm_fwd_persistent_kernel<ROWS, NT, 0>, grid, kBlockThreads, lds, num_cus, stream, kp, resident_err);
}
template <int ROWS, int NT>
hipError_t launch_bwd_prec(int prec, int grid, size_t lds, int num_cus, hipStream_t stream, void* kp, int* resident_err) {
  if (prec == 1) return resident_launch(lstm_bwd_persistent_kernel<ROWS, NT, 1>, grid, kBlockThreads, lds, num_cus, stream, kp, resident_err);
  if constexpr (ROWS >= 32) {
    if (prec == 2) return resident_launch(lstm_bwd_persistent_kernel<ROWS, NT, 2>, grid, kBlockThreads, lds, num_cus, stream, kp, resident_err);
  }
  if (prec != 0) return hipErrorInvalidValue;
  return resident_launch(lstm_bwd_persistent_kernel<ROWS, NT, 0>, grid, kBlockThreads, lds, num_cus, stream, kp, resident_err);
}
}  // namespace

size_t persistent_scratch_bytes_fwd(const RecShape& s) {
  return groups_bytes_max(s) + (size_t)s.ndir * (2 * state_bytes(s) + dbpart_bytes(s));
}
size_t persistent_scratch_bytes(const RecShape& s) { return persistent_scratch_bytes_fwd(s) + onehop_bytes_max(s); }

hipError_t persistent_forward(hipStream_t stream, const RecShape& s, const RecFwdDir* dirs, const int32_t* seq_lens,
                              char* scratch, unsigned* err, int* resident_err, int s_begin, int s_end) {
  if (s_begin < 0 || s_end > s.T || s_begin >= s_end) return hipErrorInvalidValue;
  DeviceInfo di;
  hipError_t e = device_info(&di);
  if (e != hipSuccess) return e;
  const Plan pl = make_plan(s, di.num_cus, di.max_lds);
  if (!pl.ok) { *resident_err = 1; return hipErrorInvalidValue; }
  const size_t wbytes = (size_t)pl.nchF * 1024;
  const GroupBytes gb = group_bytes(s, pl.nb);
  if (2 * 4 * wbytes > gb.exch) return hipErrorInvalidValue;
  PrepParams pp{};
  PFwdParams kp{};
  for (int g = 0; g < pl.NG; ++g) {
    char* base = scratch + (size_t)g * gb.total;
    kp.flags[g] = reinterpret_cast<unsigned*>(base);
    kp.hx[g] = base + kFlagBytes;
    pp.hx1[g] = base + kFlagBytes + 4 * wbytes;
  }
  for (int d = 0; d < s.ndir; ++d) {
    pp.h0[d] = dirs[d].h0;
    PFwdDir& k = kp.d[d];
    k.zg = dirs[d].zg; k.R = dirs[d].R; k.h0 = dirs[d].h0; k.c0 = dirs[d].c0;
    k.y = dirs[d].y; k.c = dirs[d].c; k.hT = dirs[d].hT; k.cT = dirs[d].cT;
    k.hstate = dir_array(scratch, s, d, 0); k.cstate = dir_array(scratch, s, d, 1);
    k.direction = dirs[d].direction;
  }
  pp.zero_words = reinterpret_cast<unsigned*>(scratch); pp.nzero = (size_t)pl.NG * gb.total / 4;
  pp.ndir = s.ndir; pp.B = s.B; pp.Bg = pl.Bg; pp.H = s.H; pp.KW = pl.Hp / 4; pp.wbytes = (int)wbytes; pp.MT = pl.MT; pp.prec = pl.prec;
  kp.ndir = s.ndir; kp.NG = pl.NG; kp.Bg = pl.Bg;
  kp.seq_lens = seq_lens; kp.err = err; kp.wait_ticks = g_wait_ticks; kp.mute_wg = g_mute_wg;
  kp.slow_wg = g_slow_wg; kp.slow_ticks = g_slow_ticks;
  kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy; kp.Gf = pl.Gf; kp.Hp = pl.Hp; kp.nch = pl.nchF;
  kp.s_begin = s_begin; kp.s_end = s_end;
  if (s_begin == 0) {
    hipLaunchKernelGGL(prep_kernel, dim3(256), dim3(256), 0, stream, pp);
    if (pp.h0[0] || (s.ndir > 1 && pp.h0[1])) {
      const size_t bh = (size_t)s.B * s.H;
      hipLaunchKernelGGL(seed_h0_kernel, dim3((unsigned)((bh + 255) / 256)), dim3(256), 0, stream, pp);
    }
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int grid = pl.Gf * pl.NG;
#define RLSTM_FWD_CASE(ROWS_, NT_)                                                                       \
  if (pl.ROWS == ROWS_ && pl.NT == NT_) {                                                                \
    return launch_fwd_prec<ROWS_, NT_>(pl.prec, grid, pl.ldsF, di.num_cus, stream, &kp, resident_err);   \
  }
  RLSTM_FWD_CASE(16, 1) RLSTM_FWD_CASE(32, 1) RLSTM_FWD_CASE(48, 1) RLSTM_FWD_CASE(64, 1)
  RLSTM_FWD_CASE(8, 2) RLSTM_FWD_CASE(16, 2) RLSTM_FWD_CASE(32, 2) RLSTM_FWD_CASE(48, 2) RLSTM_FWD_CASE(64, 2)
  RLSTM_FWD_CASE(8, 4) RLSTM_FWD_CASE(16, 4)
#undef RLSTM_FWD_CASE
  return hipErrorInvalidValue;
}

namespace {
// the backward pass with one exchange per step (see lstm_bwd_onehop_kernel)
hipError_t onehop_backward(hipStream_t stream, const RecShape& s, const Plan& pl, const DeviceInfo& di, const RecBwdDir* dirs,
                           const int32_t* seq_lens, char* scratch, unsigned* err, int* resident_err, int s_begin, int s_end) {
  const GroupBytes gb = group_bytes(s, pl.nb);
  if ((size_t)pl.NG * pl.px_bytes > onehop_bytes_max(s)) return hipErrorInvalidValue;
  char* pxbase = scratch + persistent_scratch_bytes_fwd(s);
  PrepParams pp{};
  PBwd1Params kp{};
  for (int g = 0; g < pl.NG; ++g) {
    kp.flags[g] = reinterpret_cast<unsigned*>(scratch + (size_t)g * gb.total);
    kp.px[g] = reinterpret_cast<float*>(pxbase + (size_t)g * pl.px_bytes);
  }
  DbSumParams ds{};
  for (int d = 0; d < s.ndir; ++d) {
    PBwdDir& k = kp.d[d];
    k.zg = dirs[d].zg; k.R = dirs[d].R; k.c = dirs[d].c; k.c0 = dirs[d].c0; k.dy = dirs[d].dy;
    k.dhT = dirs[d].dhT; k.dcT = dirs[d].dcT; k.dh0 = dirs[d].dh0; k.dc0 = dirs[d].dc0; k.db = dirs[d].db;
    k.dhstate = dir_array(scratch, s, d, 0); k.dcstate = dir_array(scratch, s, d, 1);
    k.dbpart = dir_array(scratch, s, d, 2);
    k.direction = dirs[d].direction;
    ds.db[d] = dirs[d].db; ds.dbpart[d] = k.dbpart;
  }
  // only the flags have to start at zero: every read of the exchange array is gated by them
  pp.zero_words = reinterpret_cast<unsigned*>(scratch); pp.nzero = (size_t)pl.NG * gb.total / 4;
  kp.ndir = s.ndir; kp.NG = pl.NG; kp.Bg = pl.Bg;
  kp.seq_lens = seq_lens; kp.err = err; kp.wait_ticks = g_wait_ticks; kp.mute_wg = g_mute_wg;
  kp.slow_wg = g_slow_wg; kp.slow_ticks = g_slow_ticks;
  kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy; kp.Gm = pl.Gf;
  kp.s_begin = s_begin; kp.s_end = s_end;
  if (s_begin == 0) hipLaunchKernelGGL(prep_kernel, dim3(256), dim3(256), 0, stream, pp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int grid = pl.Gf * pl.NG;
  e = hipErrorInvalidValue;
#define RLSTM_BWD1_CASE(NT_, TN_)                                                                              \
  if (pl.NT == NT_ && pl.TN == TN_)                                                                            \
    e = resident_launch(lstm_bwd_onehop_kernel<NT_, TN_>, grid, kBlockThreads, pl.ldsB1, di.num_cus, stream,   \
                        &kp, resident_err);
  RLSTM_BWD1_CASE(1, 1) RLSTM_BWD1_CASE(1, 2) RLSTM_BWD1_CASE(1, 4)
  RLSTM_BWD1_CASE(2, 1) RLSTM_BWD1_CASE(2, 2) RLSTM_BWD1_CASE(2, 4) RLSTM_BWD1_CASE(2, 8)
  RLSTM_BWD1_CASE(4, 1) RLSTM_BWD1_CASE(4, 2) RLSTM_BWD1_CASE(4, 4) RLSTM_BWD1_CASE(4, 8)
#undef RLSTM_BWD1_CASE
  if (e != hipSuccess) return e;
  if (pl.nb > 1 && s_end == s.T) {
    ds.ndir = s.ndir; ds.nb = (s.B + pl.Bg - 1) / pl.Bg; ds.n = 4 * s.H;
    hipLaunchKernelGGL(db_sum_kernel, dim3((unsigned)((ds.n + 255) / 256)), dim3(256), 0, stream, ds);
    e = hipGetLastError();
  }
  return e;
}
}  // namespace

hipError_t persistent_backward(hipStream_t stream, const RecShape& s, const RecBwdDir* dirs, const int32_t* seq_lens,
                               char* scratch, unsigned* err, int* resident_err, int s_begin, int s_end) {
  if (s_begin < 0 || s_end > s.T || s_begin >= s_end) return hipErrorInvalidValue;
  DeviceInfo di;
  hipError_t e = device_info(&di);
  if (e != hipSuccess) return e;
  const Plan pl = make_plan(s, di.num_cus, di.max_lds);
  if (!pl.ok) { *resident_err = 1; return hipErrorInvalidValue; }
  if (pl.onehop) return onehop_backward(stream, s, pl, di, dirs, seq_lens, scratch, err, resident_err, s_begin, s_end);
  const size_t wbytes = (size_t)pl.nchB * 1024;
  const size_t exch_bytes = 2 * 16 * wbytes;
  const size_t part_words = (size_t)2 * pl.PG * 4 * pl.Bp * pl.UG;
  const GroupBytes gb = group_bytes(s, pl.nb);
  if (exch_bytes > gb.exch || part_words * sizeof(unsigned long long) > gb.part) return hipErrorInvalidValue;
  PrepParams pp{};
  PBwdParams kp{};
  for (int g = 0; g < pl.NG; ++g) {
    char* base = scratch + (size_t)g * gb.total;
    kp.flags[g] = reinterpret_cast<unsigned*>(base);
    kp.dzx[g] = base + kFlagBytes;
    kp.part[g] = reinterpret_cast<unsigned long long*>(base + kFlagBytes + gb.exch);
  }
  DbSumParams ds{};
  for (int d = 0; d < s.ndir; ++d) {
    PBwdDir& k = kp.d[d];
    k.zg = dirs[d].zg; k.R = dirs[d].R; k.c = dirs[d].c; k.c0 = dirs[d].c0; k.dy = dirs[d].dy;
    k.dhT = dirs[d].dhT; k.dcT = dirs[d].dcT; k.dh0 = dirs[d].dh0; k.dc0 = dirs[d].dc0; k.db = dirs[d].db;
    k.dhstate = dir_array(scratch, s, d, 0); k.dcstate = dir_array(scratch, s, d, 1);
    k.dbpart = dir_array(scratch, s, d, 2);
    k.direction = dirs[d].direction;
    ds.db[d] = dirs[d].db; ds.dbpart[d] = k.dbpart;
  }
  pp.zero_words = reinterpret_cast<unsigned*>(scratch); pp.nzero = (size_t)pl.NG * gb.total / 4;
  pp.ndir = s.ndir;
  kp.ndir = s.ndir; kp.NG = pl.NG; kp.Bg = pl.Bg;
  kp.seq_lens = seq_lens; kp.err = err; kp.wait_ticks = g_wait_ticks; kp.mute_wg = g_mute_wg;
  kp.slow_wg = g_slow_wg; kp.slow_ticks = g_slow_ticks;
  kp.T = s.T; kp.B = s.B; kp.H = s.H; kp.ldy = s.ldy; kp.PG = pl.PG; kp.Hq = pl.Hq; kp.nch = pl.nchB;
  kp.s_begin = s_begin; kp.s_end = s_end;
  if (s_begin == 0) hipLaunchKernelGGL(prep_kernel, dim3(256), dim3(256), 0, stream, pp);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int grid = pl.Gb * pl.NG;
  e = hipErrorInvalidValue;
#define RLSTM_BWD_CASE(ROWS_, NT_)                                                                       \
  if (pl.ROWS == ROWS_ && pl.NT == NT_) {                                                                \
    e = launch_bwd_prec<ROWS_, NT_>(pl.prec, grid, pl.ldsB, di.num_cus, stream, &kp, resident_err);      \
  }
  RLSTM_BWD_CASE(16, 1) RLSTM_BWD_CASE(32, 1) RLSTM_BWD_CASE(48, 1) RLSTM_BWD_CASE(64, 1)
  RLSTM_BWD_CASE(8, 2) RLSTM_BWD_CASE(16, 2) RLSTM_BWD_CASE(32, 2) RLSTM_BWD_CASE(48, 2) RLSTM_BWD_CASE(64, 2)
  RLSTM_BWD_CASE(8, 4) RLSTM_BWD_CASE(16, 4)
#undef RLSTM_BWD_CASE
  if (e != hipSuccess) return e;
  if (pl.nb > 1 && s_end == s.T) {
    // the groups of sequences that exist: group g holds sequences [g*Bg, ...)
    ds.ndir = s.ndir; ds.nb = (s.B + pl.Bg - 1) / pl.Bg; ds.n = 4 * s.H;
    hipLaunchKernelGGL(db_sum_kernel, dim3((unsigned)((ds.n + 255) / 256)), dim3(256), 0, stream, ds);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace rlstm
