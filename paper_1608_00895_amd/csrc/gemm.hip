// Dense fp32 products on the CDNA4 matrix cores (v_mfma_f32_32x32x2_f32).
//
// These serve the whole-minibatch products of the LSTM layer (Sec. 4.2 of the
// RETURNN paper): the input projection Z = X W + b over all T*B frames, and
// after the pass back through time dX = dZ W^T, dW = X^T dZ, dR = Hprev^T dZ.
//
// Tiling: a 256-thread workgroup (4 wavefronts of 64 lanes, 2 x 2) owns a
// 128 x 128 tile of C; every wavefront owns 64 x 64 of it as 2 x 2 MFMA tiles
// of 32 x 32 (64 accumulator registers per lane).  K is consumed in slabs of
// BK; both operand slabs are staged in LDS k-major ([BK][128+pad]) so that the
// MFMA operand fetch (lane l reads element [k + l/32][l%32]) is a conflict-free
// ds_read_b32, and double-buffered so global loads of slab i+1 overlap the
// MFMAs of slab i.  Operands that are k-contiguous in memory are transposed on
// their way into LDS.
//
// Split-K (for the weight gradients, whose K = T*B is 32x larger than M or N)
// writes per-slice partial tiles to scratch and sums them in slice order in a
// second kernel, so results are bit-reproducible run to run.
#include "rlstm_internal.h"

#include <type_traits>
#include <algorithm>

namespace rlstm {

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int TM = 128;       // C tile rows per workgroup
constexpr int TN = 128;       // C tile cols per workgroup
constexpr int LDS_PAD = 4;    // floats; keeps float4 rows 16-byte aligned
constexpr int LDT = TM + LDS_PAD;

struct GemmP {
  int M, N, K;
  const float* A; int lda;
  const float* B; int ldb;
  float* C; int ldc;
  const float* bias;
  int accumulate;
  int tiles_n;
  int band_m;          // tile rows per band of the tile numbering (see tile_coords)
  int tiles;           // output tiles (tiles_m * tiles_n)
  int work;            // tiles * split-K slices: work items of the launch
  int per_xcd;         // ceil(work / 8); the grid is 8 * per_xcd workgroups
  int kchunk;          // K range per split-K slice (multiple of BK)
  float* partial;      // split-K scratch [slices][M][N] or null
  // bf16 copies of A and B (same shapes and row strides, in elements), for the kernel that takes its operands
  // as bf16 from memory; null otherwise
  const unsigned short* A16; const unsigned short* B16;
};

// Work item of a workgroup.  The dispatcher deals consecutive workgroups out to the 8 XCDs in
// turn, each with its own L2.  Workgroup i therefore takes item (i % 8) * per_xcd + i / 8: every
// XCD works through one contiguous range of items (n fastest, then m, then K slice), so the
// operand panels that neighbouring tiles share are fetched into one L2 instead of all eight.
__device__ __forceinline__ bool work_item(const GemmP& p, int* tile, int* kz) {
  const int i = blockIdx.x;
  const int item = (i & 7) * p.per_xcd + (i >> 3);
  if ((i >> 3) >= p.per_xcd || item >= p.work) return false;
  *kz = item / p.tiles;
  *tile = item - *kz * p.tiles;
  return true;
}

// Tile index -> tile coordinates.  Tiles are numbered in BANDS of band_m tile rows, column by column inside a band, so
// that the 32 tiles an XCD's CUs work on at a time form a block of band_m x (32 / band_m) tiles: they share band_m
// panels of A, which stay in the XCD's L2 for the whole band, and each panel of B is fetched once per band.  Numbered
// row by row, 32 tiles of a wide product span two whole tile rows and all of B is fetched once per two rows: counted
// at config 3, bands of 4 rows fetch 25 % less for the projections and 28 % less for the weight gradients.  band_m
// is 4 where there are 8 or more tile columns, otherwise as many rows as make 32 tiles (which is the row-by-row order).
__device__ __forceinline__ void tile_coords(const GemmP& p, int tile, int tiles_m, int* tm, int* tn) {
  const int per_band = p.band_m * p.tiles_n;
  const int band = tile / per_band;
  const int local = tile - band * per_band;
  const int hb = min(p.band_m, tiles_m - band * p.band_m);
  *tn = local / hb;
  *tm = band * p.band_m + (local - *tn * hb);
}

// Epilogue of the MFMA kernels with 32 x 32 accumulator tiles: register r of lane l holds
// C[(r/4)*8 + (l/32)*4 + r%4][l%32] of its tile.  A wavefront owns WM x WN such tiles starting at (row0, col0).
// The stores go ROW BY ROW: those of one row's 32 * WN columns are issued back to back, so that memory sees runs of
// 128 * WN bytes instead of single 128-byte pieces 4 * ldc bytes apart (measured on 96000 x 4000 outputs of the
// 256 x 256 tile kernel: 4.3 against 1.9 TB/s of stores, 817 against 654 TFLOP/s at K = 2000).
template <int WM, int WN>
__device__ __forceinline__ void store_tiles(const GemmP& p, int kz, const floatx16 (&acc)[WM][WN], int row0, int col0) {
  const int lane = threadIdx.x & 63, l32 = lane & 31, lh = lane >> 5;
  float* Cout = p.C;
  int ldc = p.ldc;
  const bool partial = p.partial != nullptr;
  if (partial) { Cout = p.partial + (size_t)kz * p.M * p.N; ldc = p.N; }
  float bv[WN];
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int col = col0 + j * 32 + l32;
    bv[j] = (!partial && p.bias && col < p.N) ? p.bias[col] : 0.f;
  }
#pragma unroll
  for (int i = 0; i < WM; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = row0 + i * 32 + (r >> 2) * 8 + lh * 4 + (r & 3);
      if (row >= p.M) continue;
      float* drow = Cout + (size_t)row * ldc + col0 + l32;
#pragma unroll
      for (int j = 0; j < WN; ++j) {
        if (col0 + j * 32 + l32 < p.N) {
          float v = acc[i][j][r] + bv[j];
          if (!partial && p.accumulate) v += drow[j * 32];
          drow[j * 32] = v;
        }
      }
    }
  }
}

// ---- slab loaders: global -> registers -> LDS ------------------------------

// "natural": element (k, mn) at ptr[k*ld + mn]; slab is BK rows of 128 floats.
template <int BK, bool VEC>
__device__ __forceinline__ void load_natural(const float* __restrict__ ptr, int ld, int k0, int kend,
                                             int mn0, int MN, float4 (&r)[BK / 8]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < BK / 8; ++i) {
    const int idx = tid + i * 256;
    const int row = idx >> 5, c4 = idx & 31;
    const int k = k0 + row, mn = mn0 + c4 * 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k < kend) {
      const float* q = ptr + (size_t)k * ld + mn;
      if (VEC) {
        if (mn < MN) v = *reinterpret_cast<const float4*>(q);
      } else {
        if (mn + 0 < MN) v.x = q[0];
        if (mn + 1 < MN) v.y = q[1];
        if (mn + 2 < MN) v.z = q[2];
        if (mn + 3 < MN) v.w = q[3];
      }
    }
    r[i] = v;
  }
}
template <int BK>
__device__ __forceinline__ void store_natural(float* __restrict__ s, const float4 (&r)[BK / 8]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < BK / 8; ++i) {
    const int idx = tid + i * 256;
    const int row = idx >> 5, c4 = idx & 31;
    *reinterpret_cast<float4*>(s + row * LDT + c4 * 4) = r[i];
  }
}

// "transposing": element (mn, k) at ptr[mn*ld + k]; slab is 128 rows of BK floats.
template <int BK, bool VEC>
__device__ __forceinline__ void load_transposing(const float* __restrict__ ptr, int ld, int k0, int kend,
                                                 int mn0, int MN, float4 (&r)[BK / 8]) {
  constexpr int QPR = BK / 4;   // float4 per row
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < BK / 8; ++i) {
    const int idx = tid + i * 256;
    const int mn = mn0 + idx / QPR, k = k0 + (idx % QPR) * 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (mn < MN) {
      const float* q = ptr + (size_t)mn * ld + k;
      if (VEC) {
        if (k < kend) v = *reinterpret_cast<const float4*>(q);
      } else {
        if (k + 0 < kend) v.x = q[0];
        if (k + 1 < kend) v.y = q[1];
        if (k + 2 < kend) v.z = q[2];
        if (k + 3 < kend) v.w = q[3];
      }
    }
    r[i] = v;
  }
}
template <int BK>
__device__ __forceinline__ void store_transposing(float* __restrict__ s, const float4 (&r)[BK / 8]) {
  constexpr int QPR = BK / 4;
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < BK / 8; ++i) {
    const int idx = tid + i * 256;
    const int mn = idx / QPR, kq = (idx % QPR) * 4;
    s[(kq + 0) * LDT + mn] = r[i].x;
    s[(kq + 1) * LDT + mn] = r[i].y;
    s[(kq + 2) * LDT + mn] = r[i].z;
    s[(kq + 3) * LDT + mn] = r[i].w;
  }
}

// TA: A stored [K,M] (natural loader); !TA: A stored [M,K] (transposing loader)
// TB: B stored [N,K] (transposing loader); !TB: B stored [K,N] (natural loader)
template <int BK, bool TA, bool TB, bool VEC>
__global__ __launch_bounds__(256) void gemm_mfma_f32_kernel(GemmP p) {
  extern __shared__ __align__(16) float smem[];
  float* As = smem;                       // [2][BK][LDT]
  float* Bs = smem + 2 * BK * LDT;        // [2][BK][LDT]

  int tile, kz;
  if (!work_item(p, &tile, &kz)) return;
  int tm, tn;
  tile_coords(p, tile, p.tiles / p.tiles_n, &tm, &tn);
  const int m0 = tm * TM, n0 = tn * TN;
  const int kbeg = kz * p.kchunk;
  const int kend = min(p.K, kbeg + p.kchunk);
  const int nslab = (kend - kbeg + BK - 1) / BK;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float4 ra[BK / 8], rb[BK / 8];
  auto loadA = [&](int k0) {
    if (TA) load_natural<BK, VEC>(p.A, p.lda, k0, kend, m0, p.M, ra);
    else    load_transposing<BK, VEC>(p.A, p.lda, k0, kend, m0, p.M, ra);
  };
  auto loadB = [&](int k0) {
    if (TB) load_transposing<BK, VEC>(p.B, p.ldb, k0, kend, n0, p.N, rb);
    else    load_natural<BK, VEC>(p.B, p.ldb, k0, kend, n0, p.N, rb);
  };
  auto storeAB = [&](int buf) {
    if (TA) store_natural<BK>(As + buf * BK * LDT, ra); else store_transposing<BK>(As + buf * BK * LDT, ra);
    if (TB) store_transposing<BK>(Bs + buf * BK * LDT, rb); else store_natural<BK>(Bs + buf * BK * LDT, rb);
  };

  if (nslab > 0) {
    loadA(kbeg); loadB(kbeg);
    storeAB(0);
  }
  __syncthreads();

  for (int s = 0; s < nslab; ++s) {
    const int buf = s & 1;
    if (s + 1 < nslab) { loadA(kbeg + (s + 1) * BK); loadB(kbeg + (s + 1) * BK); }
    const float* as = As + buf * BK * LDT + wm * 64 + l32;
    const float* bs = Bs + buf * BK * LDT + wn * 64 + l32;
    // operand fragments of step kk+2 are fetched from LDS before the MFMAs of step kk are issued
    float a0 = as[lh * LDT], a1 = as[lh * LDT + 32], b0 = bs[lh * LDT], b1 = bs[lh * LDT + 32];
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
      if (kk + 2 < BK) {
        na0 = as[(kk + 2 + lh) * LDT];
        na1 = as[(kk + 2 + lh) * LDT + 32];
        nb0 = bs[(kk + 2 + lh) * LDT];
        nb1 = bs[(kk + 2 + lh) * LDT + 32];
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads above ahead of this step's MFMAs
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
      a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
    }
    if (s + 1 < nslab) storeAB(buf ^ 1);
    __syncthreads();
  }

  store_tiles<2, 2>(p, kz, acc, m0 + wm * 64, n0 + wn * 64);
}

// ---------------------------------------------------------------------------
// The same kernel on the SHORT matrix instruction (v_mfma_f32_16x16x4_f32, 32 cycles, against the 64 cycles of
// v_mfma_f32_32x32x2_f32; the same flops per cycle), for the products that share their CUs with the persistent
// recurrent kernels.  The idea was that a recurrent wavefront, however high its priority, cannot issue its own short,
// dependent matrix instructions while one of the product's is in the pipeline.  Measured on the 4 x 500 stack the
// recurrent steps beside the products do NOT get faster (5.66 / 8.23 us against 5.62 / 8.30 us; alone 4.57 / 5.48):
// the matrix pipeline is not where the two kernels collide.  The products themselves run 4 to 10 % faster beside the
// chain (weight gradients 83 against 80 TFLOP/s, 59.2 against 60.0 ms per training pass), which is why it is kept.
// Requesting enough LDS that only one product workgroup fits beside a recurrent one changed nothing either.
// Same tiles, same LDS layout and loaders; a wavefront's 64 x 64 is 4 x 4 tiles of 16 x 16 (64 accumulator registers
// as before); per step of 4 k it reads 4 + 4 operand words from LDS for 16 instructions, the same words per k as the
// kernel above.
typedef float floatx4s __attribute__((ext_vector_type(4)));
template <int BK, bool TA, bool TB, bool VEC>
__global__ __launch_bounds__(256) void gemm_mfma_f32_short_kernel(GemmP p) {
  extern __shared__ __align__(16) float smem[];
  float* As = smem;                       // [2][BK][LDT]
  float* Bs = smem + 2 * BK * LDT;        // [2][BK][LDT]

  int tile, kz;
  if (!work_item(p, &tile, &kz)) return;
  int tm, tn;
  tile_coords(p, tile, p.tiles / p.tiles_n, &tm, &tn);
  const int m0 = tm * TM, n0 = tn * TN;
  const int kbeg = kz * p.kchunk;
  const int kend = min(p.K, kbeg + p.kchunk);
  const int nslab = (kend - kbeg + BK - 1) / BK;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l16 = lane & 15, lq = lane >> 4;

  floatx4s acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = floatx4s{0.f, 0.f, 0.f, 0.f};

  float4 ra[BK / 8], rb[BK / 8];
  auto loadA = [&](int k0) {
    if (TA) load_natural<BK, VEC>(p.A, p.lda, k0, kend, m0, p.M, ra);
    else    load_transposing<BK, VEC>(p.A, p.lda, k0, kend, m0, p.M, ra);
  };
  auto loadB = [&](int k0) {
    if (TB) load_transposing<BK, VEC>(p.B, p.ldb, k0, kend, n0, p.N, rb);
    else    load_natural<BK, VEC>(p.B, p.ldb, k0, kend, n0, p.N, rb);
  };
  auto storeAB = [&](int buf) {
    if (TA) store_natural<BK>(As + buf * BK * LDT, ra); else store_transposing<BK>(As + buf * BK * LDT, ra);
    if (TB) store_transposing<BK>(Bs + buf * BK * LDT, rb); else store_natural<BK>(Bs + buf * BK * LDT, rb);
  };

  if (nslab > 0) {
    loadA(kbeg); loadB(kbeg);
    storeAB(0);
  }
  __syncthreads();

  for (int s = 0; s < nslab; ++s) {
    const int buf = s & 1;
    if (s + 1 < nslab) { loadA(kbeg + (s + 1) * BK); loadB(kbeg + (s + 1) * BK); }
    // lane (l16, lq) holds A[row l16][k + lq] and B[k + lq][column l16] of each 16 x 16 tile
    const float* as = As + buf * BK * LDT + lq * LDT + wm * 64 + l16;
    const float* bs = Bs + buf * BK * LDT + lq * LDT + wn * 64 + l16;
    float a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = as[i * 16]; b[i] = bs[i * 16]; }
#pragma unroll
    for (int kk = 0; kk < BK; kk += 4) {
      float na[4] = {0.f, 0.f, 0.f, 0.f}, nb[4] = {0.f, 0.f, 0.f, 0.f};
      if (kk + 4 < BK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { na[i] = as[(kk + 4) * LDT + i * 16]; nb[i] = bs[(kk + 4) * LDT + i * 16]; }
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads above ahead of this step's MFMAs
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], b[j], acc[i][j], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = na[i]; b[i] = nb[i]; }
    }
    if (s + 1 < nslab) storeAB(buf ^ 1);
    __syncthreads();
  }

  // Register r of lane (l16, lq) holds C[4 * lq + r][l16] of its 16 x 16 tile.  Row by row, as in store_tiles.
  float* Cout = p.C;
  int ldc = p.ldc;
  const bool partial = p.partial != nullptr;
  if (partial) { Cout = p.partial + (size_t)kz * p.M * p.N; ldc = p.N; }
  const int col0 = n0 + wn * 64 + l16;
  float bv[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) bv[j] = (!partial && p.bias && col0 + j * 16 < p.N) ? p.bias[col0 + j * 16] : 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = m0 + wm * 64 + i * 16 + lq * 4 + r;
      if (row >= p.M) continue;
      float* drow = Cout + (size_t)row * ldc + col0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (col0 + j * 16 < p.N) {
          float v = acc[i][j][r] + bv[j];
          if (!partial && p.accumulate) v += drow[j * 16];
          drow[j * 16] = v;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Pipelined fp32 kernel for operands whose rows are whole, 16-byte aligned float4s (the usual case).
// Same tile shape as above; what differs is how a slab gets from memory into LDS:
//  * buffer loads with a byte range instead of branches: a lane outside the matrix (row or column tail,
//    K tail, slab beyond the last) gets an offset beyond the range and reads zeros;
//  * the loads of slab s+2 and the LDS stores of slab s+1 are spread over the MFMA steps of slab s, so a
//    wavefront keeps the matrix core fed by itself instead of relying on other wavefronts to cover a
//    bulk transition between slabs;
//  * an operand that is k-contiguous in memory stays k-contiguous in LDS ([128 rows][16 k], one 16-byte
//    store per float4, chunks XOR-swizzled by row so that stores and 16-byte reads are conflict-free).
//    The MFMA sums over k in any order as long as both operands agree: step j of a slab takes
//    k = 8 * (lane / 32) + j, so a lane's eight k values of a row are two 16-byte reads.
// ---------------------------------------------------------------------------
constexpr int BK2 = 16;
constexpr int SLAB_FLOATS = BK2 * LDT;             // also covers the k-contiguous form (128 * 16)
constexpr unsigned kOutOfRange = 0x80000000u;      // beyond any num_records this kernel sets (< 2^31)
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ floatx4 buffer_load_x4(__amdgpu_buffer_rsrc_t rsrc, unsigned off) {
  return __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0));
}

// chunk (16 bytes = 4 k) kq of row r of a k-contiguous slab sits at float offset:
__device__ __forceinline__ int kc_offset(int r, int kq) { return (r * 4 + (kq ^ ((r >> 1) & 3))) * 4; }

// One operand's side of the pipeline.  KC: k-contiguous in memory (A [M,K] or B stored [N,K]).
template <bool KC>
struct SlabFeeder {
  __amdgpu_buffer_rsrc_t rsrc;
  unsigned voff[2];     // byte offset of this thread's two float4s within slab 0 (or kOutOfRange)
  unsigned step;        // byte advance per slab
  int lds_off[2];       // float offset of the two float4s inside a slab buffer
  int kq4[2];           // KC: first k (relative to the slab) of each float4
  int klen;             // kend - kbeg
  floatx4 r[2];

  __device__ __forceinline__ void init(const float* ptr, int ld, int mn0, int MN, int kbeg, int kend) {
    const int tid = threadIdx.x;
    klen = kend - kbeg;
    if (KC) {
      const int rows = min(TM, MN - mn0);
      const float* base = ptr + (size_t)mn0 * ld + kbeg;
      rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, (int)((size_t)rows * ld * 4 - (size_t)kbeg * 4), 0x00020000);
      step = BK2 * 4;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int idx = tid + i * 256;
        const int row = idx >> 2, kq = idx & 3;
        voff[i] = (unsigned)row * (unsigned)ld * 4u + kq * 16u;      // rows beyond the matrix fall outside num_records
        kq4[i] = kq * 4;
        lds_off[i] = kc_offset(row, kq);
      }
    } else {
      const float* base = ptr + (size_t)kbeg * ld + mn0;
      rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, (int)((size_t)klen * ld * 4), 0x00020000);
      step = (unsigned)BK2 * (unsigned)ld * 4u;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int idx = tid + i * 256;
        const int row = idx >> 5, c4 = idx & 31;
        voff[i] = (mn0 + c4 * 4 < MN) ? (unsigned)row * (unsigned)ld * 4u + c4 * 16u : kOutOfRange;   // k tail: num_records
        kq4[i] = 0;
        lds_off[i] = row * LDT + c4 * 4;
      }
    }
  }
  // issue the loads of slab s (any s >= 0; slabs beyond the last read zeros)
  __device__ __forceinline__ void load(int s) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      unsigned off = voff[i] + (unsigned)s * step;
      if (KC) off = (s * BK2 + kq4[i] < klen) ? off : kOutOfRange;
      if (!KC) off = (s * BK2 < klen) ? off : kOutOfRange;       // keeps s * step from wrapping around
      r[i] = buffer_load_x4(rsrc, off);
    }
  }
  __device__ __forceinline__ void store(float* slab) const {
#pragma unroll
    for (int i = 0; i < 2; ++i) *reinterpret_cast<floatx4*>(slab + lds_off[i]) = r[i];
  }
};

// fragments of a k-contiguous slab for one wavefront: its two 32-row tiles, eight k per lane
__device__ __forceinline__ void read_kc(const float* slab, int row0, int l32, int lh, float (&f)[2][8]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = row0 + i * 32 + l32;
    const floatx4 lo = *reinterpret_cast<const floatx4*>(slab + kc_offset(r, 2 * lh));
    const floatx4 hi = *reinterpret_cast<const floatx4*>(slab + kc_offset(r, 2 * lh + 1));
#pragma unroll
    for (int q = 0; q < 4; ++q) { f[i][q] = lo[q]; f[i][4 + q] = hi[q]; }
  }
}

// TA: A stored [K,M]; TB: B stored [N,K] (as in the kernel above)
template <bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_mfma_f32_v2_kernel(GemmP p) {
  extern __shared__ __align__(16) float smem[];
  float* As = smem;                          // [2][SLAB_FLOATS]
  float* Bs = smem + 2 * SLAB_FLOATS;        // [2][SLAB_FLOATS]
  constexpr bool AKC = !TA, BKC = TB;

  int tile, kz;
  if (!work_item(p, &tile, &kz)) return;
  int tm, tn;
  tile_coords(p, tile, p.tiles / p.tiles_n, &tm, &tn);
  const int m0 = tm * TM, n0 = tn * TN;
  const int kbeg = kz * p.kchunk;
  const int kend = min(p.K, kbeg + p.kchunk);
  const int nslab = (kend - kbeg + BK2 - 1) / BK2;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  SlabFeeder<AKC> fa;
  SlabFeeder<BKC> fb;
  fa.init(p.A, p.lda, m0, p.M, kbeg, kend);
  fb.init(p.B, p.ldb, n0, p.N, kbeg, kend);

  fa.load(0); fb.load(0);
  fa.store(As); fb.store(Bs);
  fa.load(1); fb.load(1);
  __syncthreads();

  for (int s = 0; s < nslab; ++s) {
    const int buf = s & 1;
    const float* as = As + buf * SLAB_FLOATS;
    const float* bs = Bs + buf * SLAB_FLOATS;
    float* as_next = As + (buf ^ 1) * SLAB_FLOATS;
    float* bs_next = Bs + (buf ^ 1) * SLAB_FLOATS;
    float af[2][8], bf[2][8];
    if (AKC) read_kc(as, wm * 64, l32, lh, af);
    if (BKC) read_kc(bs, wn * 64, l32, lh, bf);
    // natural slabs: element (k, mn) at [k][mn]; this lane's k in step j is lh * 8 + j
    const float* an = as + (lh * 8) * LDT + wm * 64 + l32;
    const float* bn = bs + (lh * 8) * LDT + wn * 64 + l32;
    float a0 = 0.f, a1 = 0.f, b0 = 0.f, b1 = 0.f;
    if (!AKC) { a0 = an[0]; a1 = an[32]; }
    if (!BKC) { b0 = bn[0]; b1 = bn[32]; }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
      if (j + 1 < 8) {
        if (!AKC) { na0 = an[(j + 1) * LDT]; na1 = an[(j + 1) * LDT + 32]; }
        if (!BKC) { nb0 = bn[(j + 1) * LDT]; nb1 = bn[(j + 1) * LDT + 32]; }
      }
      // the next slab's way into LDS and the loads of the one after it, spread over the first steps
      if (j == 0) fa.store(as_next);
      if (j == 1) fb.store(bs_next);
      if (j == 2) fa.load(s + 2);
      if (j == 3) fb.load(s + 2);
      __builtin_amdgcn_sched_barrier(0);
      const float x0 = AKC ? af[0][j] : a0, x1 = AKC ? af[1][j] : a1;
      const float y0 = BKC ? bf[0][j] : b0, y1 = BKC ? bf[1][j] : b1;
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(x0, y0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(x0, y1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(x1, y0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(x1, y1, acc[1][1], 0, 0, 0);
      a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
    }
    __syncthreads();
  }

  store_tiles<2, 2>(p, kz, acc, m0 + wm * 64, n0 + wn * 64);
}

// ---------------------------------------------------------------------------
// bf16-operand variant: operands are rounded to bf16 (round to nearest even) on their way into
// LDS, products accumulate in fp32 (v_mfma_f32_32x32x16_bf16), C stays fp32.  Same 128 x 128
// tile and 2 x 2 wavefront layout; K slabs of 32.  LDS holds both operands [128][32 (+8)] bf16
// with k contiguous, because a lane's MFMA operand is 8 consecutive k of one row (one 16-byte
// ds_read).  The row stride of 40 bf16 (20 dwords) makes those reads conflict-free.
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int BKH = 32;        // K slab of the bf16 kernel
constexpr int LDK = BKH + 8;   // LDS row stride in bf16 elements

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v;
  v[0] = (__bf16)lo; v[1] = (__bf16)hi;
  return __builtin_bit_cast(unsigned, v);
}

// k-contiguous source: element (mn, k) at ptr[mn*ld + k]; slab is ROWS rows of 32 floats
template <int ROWS, bool VEC>
__device__ __forceinline__ void load_kc(const float* __restrict__ ptr, int ld, int k0, int kend, int mn0, int MN,
                                        float4 (&r)[ROWS / 32]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < ROWS / 32; ++i) {
    const int idx = tid + i * 256;
    const int mn = mn0 + (idx >> 3), k = k0 + (idx & 7) * 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (mn < MN) {
      const float* q = ptr + (size_t)mn * ld + k;
      if (VEC) {
        if (k < kend) v = *reinterpret_cast<const float4*>(q);
      } else {
        if (k + 0 < kend) v.x = q[0];
        if (k + 1 < kend) v.y = q[1];
        if (k + 2 < kend) v.z = q[2];
        if (k + 3 < kend) v.w = q[3];
      }
    }
    r[i] = v;
  }
}
template <int ROWS>
__device__ __forceinline__ void store_kc(unsigned short* __restrict__ s, const float4 (&r)[ROWS / 32]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < ROWS / 32; ++i) {
    const int idx = tid + i * 256;
    const int mn = idx >> 3, kq = (idx & 7) * 4;
    uint2 w;
    w.x = pack_bf16(r[i].x, r[i].y);
    w.y = pack_bf16(r[i].z, r[i].w);
    *reinterpret_cast<uint2*>(s + mn * LDK + kq) = w;
  }
}
// mn-contiguous source: element (k, mn) at ptr[k*ld + mn]; a work item is 2 k rows x 4 columns
template <int ROWS, bool VEC>
__device__ __forceinline__ void load_mc(const float* __restrict__ ptr, int ld, int k0, int kend, int mn0, int MN,
                                        float4 (&r)[ROWS / 32]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < ROWS / 64; ++i) {
    const int idx = tid + i * 256;
    const int mn = mn0 + (idx >> 4) * 4, k = k0 + (idx & 15) * 2;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (k + h < kend) {
        const float* q = ptr + (size_t)(k + h) * ld + mn;
        if (VEC) {
          if (mn < MN) v = *reinterpret_cast<const float4*>(q);
        } else {
          if (mn + 0 < MN) v.x = q[0];
          if (mn + 1 < MN) v.y = q[1];
          if (mn + 2 < MN) v.z = q[2];
          if (mn + 3 < MN) v.w = q[3];
        }
      }
      r[i * 2 + h] = v;
    }
  }
}
template <int ROWS>
__device__ __forceinline__ void store_mc(unsigned short* __restrict__ s, const float4 (&r)[ROWS / 32]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < ROWS / 64; ++i) {
    const int idx = tid + i * 256;
    const int mn = (idx >> 4) * 4, k = (idx & 15) * 2;
    const float4 a = r[i * 2], b = r[i * 2 + 1];
    *reinterpret_cast<unsigned*>(s + (mn + 0) * LDK + k) = pack_bf16(a.x, b.x);
    *reinterpret_cast<unsigned*>(s + (mn + 1) * LDK + k) = pack_bf16(a.y, b.y);
    *reinterpret_cast<unsigned*>(s + (mn + 2) * LDK + k) = pack_bf16(a.z, b.z);
    *reinterpret_cast<unsigned*>(s + (mn + 3) * LDK + k) = pack_bf16(a.w, b.w);
  }
}

// WM x WN: 32 x 32 MFMA tiles per wavefront; the workgroup's 2 x 2 wavefronts cover a
// (64*WM) x (64*WN) tile of C: 128 x 128 for small products, 256 x 256 where there are enough
// tiles to fill the chip (each operand byte fetched then feeds twice the MFMA work).
template <int WM, int WN, bool TA, bool TB, bool VEC>
__global__ __launch_bounds__(256) void gemm_mfma_bf16_kernel(GemmP p) {
  constexpr int TMB = 64 * WM, TNB = 64 * WN;
  extern __shared__ __align__(16) float smem[];
  unsigned short* As = reinterpret_cast<unsigned short*>(smem);     // [2][TMB][LDK]
  unsigned short* Bs = As + 2 * TMB * LDK;                          // [2][TNB][LDK]

  int tile, kz;
  if (!work_item(p, &tile, &kz)) return;
  int tm, tn;
  tile_coords(p, tile, p.tiles / p.tiles_n, &tm, &tn);
  const int m0 = tm * TMB, n0 = tn * TNB;
  const int kbeg = kz * p.kchunk;
  const int kend = min(p.K, kbeg + p.kchunk);
  const int nslab = (kend - kbeg + BKH - 1) / BKH;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float4 ra[TMB / 32], rb[TNB / 32];
  auto loadA = [&](int k0) {
    if (TA) load_mc<TMB, VEC>(p.A, p.lda, k0, kend, m0, p.M, ra); else load_kc<TMB, VEC>(p.A, p.lda, k0, kend, m0, p.M, ra);
  };
  auto loadB = [&](int k0) {
    if (TB) load_kc<TNB, VEC>(p.B, p.ldb, k0, kend, n0, p.N, rb); else load_mc<TNB, VEC>(p.B, p.ldb, k0, kend, n0, p.N, rb);
  };
  auto storeAB = [&](int buf) {
    if (TA) store_mc<TMB>(As + buf * TMB * LDK, ra); else store_kc<TMB>(As + buf * TMB * LDK, ra);
    if (TB) store_kc<TNB>(Bs + buf * TNB * LDK, rb); else store_mc<TNB>(Bs + buf * TNB * LDK, rb);
  };

  if (nslab > 0) {
    loadA(kbeg); loadB(kbeg);
    storeAB(0);
  }
  __syncthreads();

  for (int s = 0; s < nslab; ++s) {
    const int buf = s & 1;
    if (s + 1 < nslab) { loadA(kbeg + (s + 1) * BKH); loadB(kbeg + (s + 1) * BKH); }
    const unsigned short* as = As + buf * TMB * LDK + (wm * 32 * WM + l32) * LDK + lh * 8;
    const unsigned short* bs = Bs + buf * TNB * LDK + (wn * 32 * WN + l32) * LDK + lh * 8;
#pragma unroll
    for (int ks = 0; ks < BKH; ks += 16) {
      // lane l supplies row l%32, k = ks + 8*(l/32) .. +7
      bf16x8 af[WM], bfr[WN];
#pragma unroll
      for (int i = 0; i < WM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(as + i * 32 * LDK + ks);
#pragma unroll
      for (int j = 0; j < WN; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(bs + j * 32 * LDK + ks);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (s + 1 < nslab) storeAB(buf ^ 1);
    __syncthreads();
  }

  store_tiles<WM, WN>(p, kz, acc, m0 + wm * WM * 32, n0 + wn * WN * 32);
}

// ---------------------------------------------------------------------------
// fp32 product on the bf16 matrix cores.  An fp32 number is exactly the sum of three bf16 numbers (its 24
// significant bits cut into 8 + 8 + 8: x = x1 + x2 + x3, each part the leading bits of what the parts before it
// left over, |x2| < 2^-7 |x|, |x3| < 2^-15 |x|).  On their way into LDS both operands are cut this way into three
// planes; the product of two fp32 numbers is then the sum of nine bf16 products, each exact in the fp32
// accumulator's format, of which the six largest are formed (1,1) (1,2) (2,1) (2,2) (1,3) (3,1): what is left out,
// (2,3) (3,2) (3,3), is below 2^-21 |x y| per term, the size of fp32's own rounding of a sum of such terms.  Six
// v_mfma_f32_32x32x16_bf16 do the work of eight v_mfma_f32_32x32x2_f32 in 3/8 of the matrix cores' time.
// 128 x 128 tile, 2 x 2 wavefronts, K slabs of 16, LDS [2 stages][3 planes][128 rows][16 (+8)] bf16 per operand.
// Infinities turn into NaN (inf - inf in the cut), as they do in most sums of products anyway.
// ---------------------------------------------------------------------------
constexpr int BK3 = 16;         // K slab of the three-part kernel: one matrix instruction deep
constexpr int LDK3 = BK3 + 8;   // LDS row stride in bf16 (12 words: 16-byte reads of 16 consecutive rows cover all banks)
constexpr size_t gemm_3xbf16_lds_bytes() { return (size_t)2 * 3 * (128 + 128) * LDK3 * sizeof(unsigned short); }

// the three parts of two neighbouring values (a at the lower k), packed as bf16 pairs
__device__ __forceinline__ void cut3(float a, float b, unsigned& w1, unsigned& w2, unsigned& w3) {
  const unsigned a1 = __float_as_uint(a) & 0xffff0000u, b1 = __float_as_uint(b) & 0xffff0000u;
  const float ra = a - __uint_as_float(a1), rb = b - __uint_as_float(b1);             // exact
  const unsigned a2 = __float_as_uint(ra) & 0xffff0000u, b2 = __float_as_uint(rb) & 0xffff0000u;
  const float sa = ra - __uint_as_float(a2), sb = rb - __uint_as_float(b2);           // exact, at most 8 significant bits
  w1 = __builtin_amdgcn_perm(b1, a1, 0x07060302u);
  w2 = __builtin_amdgcn_perm(b2, a2, 0x07060302u);
  w3 = __builtin_amdgcn_perm(__float_as_uint(sb), __float_as_uint(sa), 0x07060302u);
}

// k-contiguous source: element (mn, k) at ptr[mn*ld + k]; a slab is ROWS rows of 16 floats, a work item 4 of them
template <int ROWS, bool VEC>
__device__ __forceinline__ void load_kc3(const float* __restrict__ ptr, int ld, int k0, int kend, int mn0, int MN,
                                         float4 (&r)[ROWS / 64]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < ROWS / 64; ++i) {
    const int idx = tid + i * 256;
    const int mn = mn0 + (idx >> 2), k = k0 + (idx & 3) * 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (mn < MN) {
      const float* q = ptr + (size_t)mn * ld + k;
      if (VEC) {
        if (k < kend) v = *reinterpret_cast<const float4*>(q);
      } else {
        if (k + 0 < kend) v.x = q[0];
        if (k + 1 < kend) v.y = q[1];
        if (k + 2 < kend) v.z = q[2];
        if (k + 3 < kend) v.w = q[3];
      }
    }
    r[i] = v;
  }
}
template <int ROWS>
__device__ __forceinline__ void store_kc3(unsigned short* __restrict__ s, const float4 (&r)[ROWS / 64]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < ROWS / 64; ++i) {
    const int idx = tid + i * 256;
    const int mn = idx >> 2, kq = (idx & 3) * 4;
    uint2 w1, w2, w3;
    cut3(r[i].x, r[i].y, w1.x, w2.x, w3.x);
    cut3(r[i].z, r[i].w, w1.y, w2.y, w3.y);
    unsigned short* q = s + mn * LDK3 + kq;
    *reinterpret_cast<uint2*>(q) = w1;
    *reinterpret_cast<uint2*>(q + ROWS * LDK3) = w2;
    *reinterpret_cast<uint2*>(q + 2 * ROWS * LDK3) = w3;
  }
}
// mn-contiguous source: element (k, mn) at ptr[k*ld + mn]; a work item is 2 k rows x 4 columns
template <int ROWS, bool VEC>
__device__ __forceinline__ void load_mc3(const float* __restrict__ ptr, int ld, int k0, int kend, int mn0, int MN,
                                         float4 (&r)[ROWS / 64]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < ROWS / 128; ++i) {
    const int idx = tid + i * 256;
    const int mn = mn0 + (idx >> 3) * 4, k = k0 + (idx & 7) * 2;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (k + h < kend) {
        const float* q = ptr + (size_t)(k + h) * ld + mn;
        if (VEC) {
          if (mn < MN) v = *reinterpret_cast<const float4*>(q);
        } else {
          if (mn + 0 < MN) v.x = q[0];
          if (mn + 1 < MN) v.y = q[1];
          if (mn + 2 < MN) v.z = q[2];
          if (mn + 3 < MN) v.w = q[3];
        }
      }
      r[i * 2 + h] = v;
    }
  }
}
template <int ROWS>
__device__ __forceinline__ void store_mc3(unsigned short* __restrict__ s, const float4 (&r)[ROWS / 64]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < ROWS / 128; ++i) {
    const int idx = tid + i * 256;
    const int mn = (idx >> 3) * 4, k = (idx & 7) * 2;
    const float4 a = r[i * 2], b = r[i * 2 + 1];
    const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      unsigned w1, w2, w3;
      cut3(av[c], bv[c], w1, w2, w3);
      unsigned short* q = s + (mn + c) * LDK3 + k;
      *reinterpret_cast<unsigned*>(q) = w1;
      *reinterpret_cast<unsigned*>(q + ROWS * LDK3) = w2;
      *reinterpret_cast<unsigned*>(q + 2 * ROWS * LDK3) = w3;
    }
  }
}

template <bool TA, bool TB, bool VEC>
__global__ __launch_bounds__(256) void gemm_f32_3xbf16_kernel(GemmP p) {
  constexpr int TMB = 128, TNB = 128;
  constexpr int PLANE = TMB * LDK3;                                  // one part of one operand's slab
  extern __shared__ __align__(16) float smem[];
  unsigned short* As = reinterpret_cast<unsigned short*>(smem);     // [2][3][TMB][LDK3]
  unsigned short* Bs = As + 2 * 3 * PLANE;                          // [2][3][TNB][LDK3]

  int tile, kz;
  if (!work_item(p, &tile, &kz)) return;
  int tm, tn;
  tile_coords(p, tile, p.tiles / p.tiles_n, &tm, &tn);
  const int m0 = tm * TMB, n0 = tn * TNB;
  const int kbeg = kz * p.kchunk;
  const int kend = min(p.K, kbeg + p.kchunk);
  const int nslab = (kend - kbeg + BK3 - 1) / BK3;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float4 ra[TMB / 64], rb[TNB / 64];
  auto load = [&](int slab) {
    const int k0 = kbeg + slab * BK3;
    if (TA) load_mc3<TMB, VEC>(p.A, p.lda, k0, kend, m0, p.M, ra); else load_kc3<TMB, VEC>(p.A, p.lda, k0, kend, m0, p.M, ra);
    if (TB) load_kc3<TNB, VEC>(p.B, p.ldb, k0, kend, n0, p.N, rb); else load_mc3<TNB, VEC>(p.B, p.ldb, k0, kend, n0, p.N, rb);
  };
  auto store = [&](int buf) {
    if (TA) store_mc3<TMB>(As + buf * 3 * PLANE, ra); else store_kc3<TMB>(As + buf * 3 * PLANE, ra);
    if (TB) store_kc3<TNB>(Bs + buf * 3 * PLANE, rb); else store_mc3<TNB>(Bs + buf * 3 * PLANE, rb);
  };

  if (nslab > 0) { load(0); store(0); }
  __syncthreads();

  for (int s = 0; s < nslab; ++s) {
    const int buf = s & 1;
    if (s + 1 < nslab) load(s + 1);
    // lane l supplies row l%32, k = 8*(l/32) .. +7
    const unsigned short* as = As + buf * 3 * PLANE + (wm * 64 + l32) * LDK3 + lh * 8;
    const unsigned short* bs = Bs + buf * 3 * PLANE + (wn * 64 + l32) * LDK3 + lh * 8;
    bf16x8 af[3][2], bfr[3][2];
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[q][i] = *reinterpret_cast<const bf16x8*>(as + q * PLANE + i * 32 * LDK3);
        bfr[q][i] = *reinterpret_cast<const bf16x8*>(bs + q * PLANE + i * 32 * LDK3);
      }
    // small terms first; the four tiles alternate so that no instruction waits for the one before it
    constexpr int QA[6] = {2, 0, 1, 1, 0, 0}, QB[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
    for (int t = 0; t < 6; ++t)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[QA[t]][i], bfr[QB[t]][j], acc[i][j], 0, 0, 0);
    if (s + 1 < nslab) store(buf ^ 1);
    __syncthreads();
  }

  store_tiles<2, 2>(p, kz, acc, m0 + wm * 64, n0 + wn * 64);
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int slices,
                                                             int M, int N, float* __restrict__ C, int ldc,
                                                             const float* __restrict__ bias, int accumulate) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t mn = (size_t)M * N;
  if (idx >= mn) return;
  float s = 0.f;
  for (int z = 0; z < slices; ++z) s += partial[(size_t)z * mn + idx];
  const int m = (int)(idx / N), n = (int)(idx % N);
  if (bias) s += bias[n];
  float* dst = C + (size_t)m * ldc + n;
  if (accumulate) s += *dst;
  *dst = s;
}

// Many slices of a small matrix (weight gradients summed over hundreds of thousands of rows): 64 outputs per
// workgroup, the slices dealt to G groups of threads in contiguous runs, the G sums added in group order.
// The order of additions depends only on the slice count, so results stay bit-reproducible.
template <int G>
__global__ __launch_bounds__(64 * G) void splitk_reduce_groups_kernel(const float* __restrict__ partial, int slices,
                                                                      int M, int N, float* __restrict__ C, int ldc,
                                                                      const float* __restrict__ bias, int accumulate) {
  __shared__ float part[G][64];
  const int o = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const size_t idx = (size_t)blockIdx.x * 64 + o;
  const size_t mn = (size_t)M * N;
  const int per = (slices + G - 1) / G;
  const int z0 = grp * per, z1 = min(slices, z0 + per);
  float s = 0.f;
  if (idx < mn)
    for (int z = z0; z < z1; ++z) s += partial[(size_t)z * mn + idx];
  part[grp][o] = s;
  __syncthreads();
  if (grp != 0 || idx >= mn) return;
  s = part[0][o];
#pragma unroll
  for (int k = 1; k < G; ++k) s += part[k][o];
  const int m = (int)(idx / N), n = (int)(idx % N);
  if (bias) s += bias[n];
  float* dst = C + (size_t)m * ldc + n;
  if (accumulate) s += *dst;
  *dst = s;
}

// sum of the split-K partial results [slices][M][N] into C
hipError_t splitk_reduce(hipStream_t stream, const float* partial, int slices, int M, int N, float* C, int ldc,
                         const float* bias, bool accumulate) {
  const size_t total = (size_t)M * N;
  const int acc = accumulate ? 1 : 0;
  if (slices >= 256 && total <= (size_t)64 * 1024)
    hipLaunchKernelGGL(splitk_reduce_groups_kernel<16>, dim3((unsigned)((total + 63) / 64)), dim3(1024), 0, stream,
                       partial, slices, M, N, C, ldc, bias, acc);
  else if (slices >= 64 && total <= (size_t)256 * 1024)
    hipLaunchKernelGGL(splitk_reduce_groups_kernel<4>, dim3((unsigned)((total + 63) / 64)), dim3(256), 0, stream,
                       partial, slices, M, N, C, ldc, bias, acc);
  else
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       partial, slices, M, N, C, ldc, bias, acc);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Tall and skinny: C[M,N] = sum_k A[k,m] B[k,n] with M <= 80, N <= 160 and K in the hundreds of thousands (the
// weight gradients of a layer with few units summed over every pixel of a batch of images).  The 128 x 128
// tiles of the kernels above would be half empty, and this product is bound by the matrix cores, not by HBM
// (24 FLOP per byte in fp32).  Here the whole of C is one tile of 5 x 10 MFMA blocks: a workgroup of ten
// wavefronts takes a slice of K, wavefront w block column w of all five block rows (5 accumulators, 6 LDS reads
// per 5 MFMAs); two workgroups a CU put five wavefronts on every SIMD, which keeps its matrix core fed (five
// wavefronts with two block columns each left the SIMDs with 3, 3, 2, 2 wavefronts and were 4 % slower).  Both
// operands are row-contiguous in k, so a chunk of 32 rows is a flat copy: HBM -> registers one chunk ahead ->
// LDS (row pitches 80 and 176 floats: the four k of an MFMA operand fall into different banks).  Partial sums
// [slices][M][N] are added by the split-K reduction above.
// ---------------------------------------------------------------------------
constexpr int TS_KC = 32;                  // rows of a chunk
constexpr int TS_MB = 5, TS_NW = 10;       // block rows; wavefronts (one block column each)
constexpr int TS_NBW = 1;                  // block columns per wavefront
constexpr int TS_PA = 16 * TS_MB;          // 80: = 16 mod 32
constexpr int TS_PB = 16 * TS_NBW * TS_NW + 16;   // 176: = 16 mod 32
constexpr int TS_THREADS = 64 * TS_NW;
constexpr int TS_NLD = (TS_KC * (TS_PA / 4 + 16 * TS_NBW * TS_NW / 4) + TS_THREADS - 1) / TS_THREADS;   // float4 per thread and chunk
struct TsP { const float* A; const float* B; float* partial; int M, N, K, lda, ldb, kchunk; };

__global__ __launch_bounds__(TS_THREADS) void tsmm_tn_f32_kernel(TsP p) {
  __shared__ __align__(16) float As[TS_KC * TS_PA];
  __shared__ __align__(16) float Bs[TS_KC * TS_PB];
  const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int M4 = p.M / 4, N4 = p.N / 4, nA = TS_KC * M4, nAB = nA + TS_KC * N4;
  const int k_begin = blockIdx.x * p.kchunk, k_end = min(p.K, k_begin + p.kchunk);

  for (int i = tid; i < TS_KC * TS_PA; i += TS_THREADS) As[i] = 0.f;   // columns beyond M, N stay zero
  for (int i = tid; i < TS_KC * TS_PB; i += TS_THREADS) Bs[i] = 0.f;

  // the float4s this thread moves per chunk: row of the chunk, offset in HBM relative to the chunk's first row, offset in LDS
  int srow[TS_NLD], slds[TS_NLD];
  long long sg[TS_NLD];
  bool sa[TS_NLD];
#pragma unroll
  for (int i = 0; i < TS_NLD; ++i) {
    const int idx = tid + i * TS_THREADS;
    sa[i] = idx < nA;
    const int j = sa[i] ? idx : idx - nA, w4 = sa[i] ? M4 : N4;
    srow[i] = idx < nAB ? j / w4 : TS_KC * 2;                          // beyond the chunk: never loaded
    const int c4 = j % w4;
    sg[i] = (long long)srow[i] * (sa[i] ? p.lda : p.ldb) + 4 * c4;
    slds[i] = srow[i] * (sa[i] ? TS_PA : TS_PB) + 4 * c4;
  }
  floatx4 st[TS_NLD];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < TS_NLD; ++i) {
      st[i] = floatx4{0.f, 0.f, 0.f, 0.f};
      if (srow[i] < TS_KC && k0 + srow[i] < k_end) {
        const float* src = sa[i] ? p.A + (size_t)k0 * p.lda + sg[i] : p.B + (size_t)k0 * p.ldb + sg[i];
        st[i] = *reinterpret_cast<const floatx4*>(src);
      }
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int i = 0; i < TS_NLD; ++i)
      if (srow[i] < TS_KC) *reinterpret_cast<floatx4*>((sa[i] ? As : Bs) + slds[i]) = st[i];
  };

  floatx4 acc[TS_MB][TS_NBW];
#pragma unroll
  for (int mb = 0; mb < TS_MB; ++mb)
#pragma unroll
    for (int nb = 0; nb < TS_NBW; ++nb) acc[mb][nb] = floatx4{0.f, 0.f, 0.f, 0.f};

  fetch(k_begin);
  for (int k0 = k_begin; k0 < k_end; k0 += TS_KC) {
    __syncthreads();                   // the chunk before has been read
    stage();
    __syncthreads();
    if (k0 + TS_KC < k_end) fetch(k0 + TS_KC);
    const float* a = As + lq * TS_PA + l16;
    const float* b = Bs + lq * TS_PB + 16 * TS_NBW * wave + l16;
#pragma unroll
    for (int j = 0; j < TS_KC / 4; ++j) {
      float av[TS_MB];
#pragma unroll
      for (int mb = 0; mb < TS_MB; ++mb) av[mb] = a[4 * j * TS_PA + 16 * mb];
      float bv[TS_NBW];
#pragma unroll
      for (int nb = 0; nb < TS_NBW; ++nb) bv[nb] = b[4 * j * TS_PB + 16 * nb];
#pragma unroll
      for (int mb = 0; mb < TS_MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < TS_NBW; ++nb)
          acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[mb], bv[nb], acc[mb][nb], 0, 0, 0);
    }
  }

  float* out = p.partial + (size_t)blockIdx.x * p.M * p.N;
#pragma unroll
  for (int mb = 0; mb < TS_MB; ++mb)
#pragma unroll
    for (int nb = 0; nb < TS_NBW; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = 16 * mb + 4 * lq + i, n = 16 * TS_NBW * wave + 16 * nb + l16;
        if (m < p.M && n < p.N) out[(size_t)m * p.N + n] = acc[mb][nb][i];
      }
}

// Plain product for the stepwise engine: one thread per element of C.
__global__ __launch_bounds__(256) void gemm_naive_kernel(GemmP p, int transA, int transB, int round_bf16) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)p.M * p.N) return;
  const int m = (int)(idx / p.N), n = (int)(idx % p.N);
  float s = 0.f;
  for (int k = 0; k < p.K; ++k) {
    float a = transA ? p.A[(size_t)k * p.lda + m] : p.A[(size_t)m * p.lda + k];
    float b = transB ? p.B[(size_t)n * p.ldb + k] : p.B[(size_t)k * p.ldb + n];
    if (round_bf16) { a = (float)(__bf16)a; b = (float)(__bf16)b; }
    s = fmaf(a, b, s);
  }
  if (p.bias) s += p.bias[n];
  float* dst = p.C + (size_t)m * p.ldc + n;
  if (p.accumulate) s += *dst;
  *dst = s;
}

inline bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

template <int BK, bool TA, bool TB>
hipError_t launch_mfma(hipStream_t stream, const GemmP& p, dim3 grid, bool vec, bool short_mfma) {
  const size_t lds = (size_t)4 * BK * LDT * sizeof(float);
  if (short_mfma) {
    if (vec) hipLaunchKernelGGL((gemm_mfma_f32_short_kernel<BK, TA, TB, true>), grid, dim3(256), lds, stream, p);
    else     hipLaunchKernelGGL((gemm_mfma_f32_short_kernel<BK, TA, TB, false>), grid, dim3(256), lds, stream, p);
  } else if (vec) {
    hipLaunchKernelGGL((gemm_mfma_f32_kernel<BK, TA, TB, true>), grid, dim3(256), lds, stream, p);
  } else {
    hipLaunchKernelGGL((gemm_mfma_f32_kernel<BK, TA, TB, false>), grid, dim3(256), lds, stream, p);
  }
  return hipGetLastError();
}

template <bool TA, bool TB>
hipError_t launch_mfma_v2(hipStream_t stream, const GemmP& p, dim3 grid) {
  const size_t lds = (size_t)4 * SLAB_FLOATS * sizeof(float);
  hipLaunchKernelGGL((gemm_mfma_f32_v2_kernel<TA, TB>), grid, dim3(256), lds, stream, p);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Pipelined form of the bf16-operand kernel (operands of whole, 16-byte aligned float4s, as for the pipelined
// fp32 kernel): the same tiles and the same LDS layout as above; the fp32 operands of slab s+2 are fetched with
// range-checked buffer loads, and rounded and stored into LDS as slab s+1, in between the MFMAs of slab s.
// A timing probe of the kernel above without its loads and LDS stores ran at 0.84-1.48 PFLOP/s against
// 0.29-0.54 with them: the bulk transition between slabs, not the matrix core, set its speed.
// ---------------------------------------------------------------------------
// One operand's side: ROWS rows of the tile, a slab of 32 k.  A unit is two float4 of one thread.
template <int ROWS, bool KC>
struct SlabFeederBf {
  static constexpr int kUnits = ROWS / 64;
  __amdgpu_buffer_rsrc_t rsrc;
  unsigned voff[kUnits][2];
  unsigned step;
  int lds_off[kUnits][2];      // KC: bf16 offset of each float4's 4 values; !KC: [u][0] = offset of the unit's first row
  int kq[kUnits][2];           // KC: first k of each float4 inside the slab
  int klen;
  floatx4 r[kUnits][2];

  __device__ __forceinline__ void init(const float* ptr, int ld, int mn0, int MN, int kbeg, int kend) {
    const int tid = threadIdx.x;
    klen = kend - kbeg;
    if (KC) {
      const int rows = min(ROWS, MN - mn0);
      const float* base = ptr + (size_t)mn0 * ld + kbeg;
      rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, (int)((size_t)rows * ld * 4 - (size_t)kbeg * 4), 0x00020000);
      step = BKH * 4;
#pragma unroll
      for (int u = 0; u < kUnits; ++u)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int idx = tid + (u * 2 + h) * 256;
          const int row = idx >> 3, q = (idx & 7) * 4;
          voff[u][h] = (unsigned)row * (unsigned)ld * 4u + q * 4u;
          kq[u][h] = q;
          lds_off[u][h] = row * LDK + q;
        }
    } else {
      const float* base = ptr + (size_t)kbeg * ld + mn0;
      rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, (int)((size_t)klen * ld * 4), 0x00020000);
      step = (unsigned)BKH * (unsigned)ld * 4u;
#pragma unroll
      for (int u = 0; u < kUnits; ++u) {
        const int idx = tid + u * 256;
        const int mn = (idx >> 4) * 4, k = (idx & 15) * 2;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          voff[u][h] = (mn0 + mn < MN) ? (unsigned)(k + h) * (unsigned)ld * 4u + mn * 4u : kOutOfRange;
          kq[u][h] = 0;
        }
        lds_off[u][0] = mn * LDK + k;
        lds_off[u][1] = 0;
      }
    }
  }
  __device__ __forceinline__ void load(int u, int s) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      unsigned off = voff[u][h] + (unsigned)s * step;
      if (KC) off = (s * BKH + kq[u][h] < klen) ? off : kOutOfRange;
      else    off = (s * BKH < klen) ? off : kOutOfRange;
      r[u][h] = buffer_load_x4(rsrc, off);
    }
  }
  __device__ __forceinline__ void store(int u, unsigned short* slab) const {
    if (KC) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        uint2 w;
        w.x = pack_bf16(r[u][h][0], r[u][h][1]);
        w.y = pack_bf16(r[u][h][2], r[u][h][3]);
        *reinterpret_cast<uint2*>(slab + lds_off[u][h]) = w;
      }
    } else {
      // rows k and k+1 of four columns: each column's pair of k is one 32-bit store
      unsigned short* q = slab + lds_off[u][0];
#pragma unroll
      for (int c = 0; c < 4; ++c) *reinterpret_cast<unsigned*>(q + c * LDK) = pack_bf16(r[u][0][c], r[u][1][c]);
    }
  }
};

// ---------------------------------------------------------------------------
// Pipelined form of the three-part kernel (gemm_f32_3xbf16_kernel): range-checked buffer loads without branches, so
// that the wait before a slab's way into LDS counts only that slab's loads; D slabs on their way from memory at any
// time (slab s waits in register stage s % D); the cutting and the LDS stores of slab s+1 and the loads of slab
// s+1+D are dealt out between the 24 matrix instructions of slab s, a few behind each (sched_group_barrier).  One such workgroup per CU, as beside the recurrent
// kernels, then keeps its matrix cores fed by itself.
// ---------------------------------------------------------------------------
template <bool KC, int D>
struct SlabFeeder3 {
  __amdgpu_buffer_rsrc_t rsrc;
  unsigned voff[2];
  unsigned step;
  int lds_off[2];              // KC: bf16 offset of each float4's 4 values; !KC: [0] = offset of (first column, k)
  int kq[2];                   // KC: first k of each float4 inside the slab
  int klen;
  floatx4 r[D][2];

  __device__ __forceinline__ void init(const float* ptr, int ld, int mn0, int MN, int kbeg, int kend) {
    const int tid = threadIdx.x;
    klen = kend - kbeg;
    if (KC) {
      const int rows = min(128, MN - mn0);
      const float* base = ptr + (size_t)mn0 * ld + kbeg;
      rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, (int)((size_t)rows * ld * 4 - (size_t)kbeg * 4), 0x00020000);
      step = BK3 * 4;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int idx = tid + h * 256;
        const int row = idx >> 2, q = (idx & 3) * 4;
        voff[h] = (unsigned)row * (unsigned)ld * 4u + q * 4u;       // rows beyond the matrix fall outside num_records
        kq[h] = q;
        lds_off[h] = row * LDK3 + q;
      }
    } else {
      const float* base = ptr + (size_t)kbeg * ld + mn0;
      rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, (int)((size_t)klen * ld * 4), 0x00020000);
      step = (unsigned)BK3 * (unsigned)ld * 4u;
      const int mn = (tid >> 3) * 4, k = (tid & 7) * 2;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        voff[h] = (mn0 + mn < MN) ? (unsigned)(k + h) * (unsigned)ld * 4u + mn * 4u : kOutOfRange;   // k tail: num_records
        kq[h] = 0;
      }
      lds_off[0] = mn * LDK3 + k;
      lds_off[1] = 0;
    }
  }
  // issue the loads of slab s into a stage (any s >= 0; slabs beyond the last read zeros)
  __device__ __forceinline__ void load(int stage, int s) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      unsigned off = voff[h] + (unsigned)s * step;
      if (KC) off = (s * BK3 + kq[h] < klen) ? off : kOutOfRange;
      else    off = (s * BK3 < klen) ? off : kOutOfRange;          // keeps s * step from wrapping around
      r[stage][h] = buffer_load_x4(rsrc, off);
    }
  }
  // cut a stage into its three parts and write them to the three planes of a slab buffer
  __device__ __forceinline__ void store(int stage, unsigned short* slab) const {
    constexpr int PLANE = 128 * LDK3;
    if (KC) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        uint2 w1, w2, w3;
        cut3(r[stage][h][0], r[stage][h][1], w1.x, w2.x, w3.x);
        cut3(r[stage][h][2], r[stage][h][3], w1.y, w2.y, w3.y);
        unsigned short* q = slab + lds_off[h];
        *reinterpret_cast<uint2*>(q) = w1;
        *reinterpret_cast<uint2*>(q + PLANE) = w2;
        *reinterpret_cast<uint2*>(q + 2 * PLANE) = w3;
      }
    } else {
      // rows k and k+1 of four columns: each column's pair of k is one 32-bit store per plane
      unsigned short* q = slab + lds_off[0];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        unsigned w1, w2, w3;
        cut3(r[stage][0][c], r[stage][1][c], w1, w2, w3);
        *reinterpret_cast<unsigned*>(q + c * LDK3) = w1;
        *reinterpret_cast<unsigned*>(q + c * LDK3 + PLANE) = w2;
        *reinterpret_cast<unsigned*>(q + c * LDK3 + 2 * PLANE) = w3;
      }
    }
  }
};

template <bool TA, bool TB, int D>
__global__ __launch_bounds__(256) void gemm_f32_3xbf16_v2_kernel(GemmP p) {
  constexpr int PLANE = 128 * LDK3;
  constexpr bool AKC = !TA, BKC = TB;
  extern __shared__ __align__(16) float smem[];
  unsigned short* As = reinterpret_cast<unsigned short*>(smem);     // [2][3][128][LDK3]
  unsigned short* Bs = As + 2 * 3 * PLANE;                          // [2][3][128][LDK3]

  int tile, kz;
  if (!work_item(p, &tile, &kz)) return;
  int tm, tn;
  tile_coords(p, tile, p.tiles / p.tiles_n, &tm, &tn);
  const int m0 = tm * 128, n0 = tn * 128;
  const int kbeg = kz * p.kchunk;
  const int kend = min(p.K, kbeg + p.kchunk);
  const int nslab = (kend - kbeg + BK3 - 1) / BK3;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  SlabFeeder3<AKC, D> fa;
  SlabFeeder3<BKC, D> fb;
  fa.init(p.A, p.lda, m0, p.M, kbeg, kend);
  fb.init(p.B, p.ldb, n0, p.N, kbeg, kend);
#pragma unroll
  for (int d = 0; d < D; ++d) { fa.load(d, d); fb.load(d, d); }
  fa.store(0, As); fb.store(0, Bs);
  fa.load(0, D); fb.load(0, D);
  __syncthreads();

  // lane l supplies row l%32, k = 8*(l/32) .. +7
  const int a_frag = (wm * 64 + l32) * LDK3 + lh * 8, b_frag = (wn * 64 + l32) * LDK3 + lh * 8;
  auto slab = [&](int s, int d) {
    const int buf = s & 1;
    const int next = (d + 1) % D;          // the stage slab s+1 waits in (a constant once the loops are unrolled)
    const unsigned short* as = As + buf * 3 * PLANE + a_frag;
    const unsigned short* bs = Bs + buf * 3 * PLANE + b_frag;
    unsigned short* as_next = As + (buf ^ 1) * 3 * PLANE;
    unsigned short* bs_next = Bs + (buf ^ 1) * 3 * PLANE;
    bf16x8 af[3][2], bfr[3][2];
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[q][i] = *reinterpret_cast<const bf16x8*>(as + q * PLANE + i * 32 * LDK3);
        bfr[q][i] = *reinterpret_cast<const bf16x8*>(bs + q * PLANE + i * 32 * LDK3);
      }
    // small terms first; the four tiles alternate so that no instruction waits for the one before it
    constexpr int QA[6] = {2, 0, 1, 1, 0, 0}, QB[6] = {0, 2, 1, 0, 1, 0};
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 6; ++t)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[QA[t]][i], bfr[QB[t]][j], acc[i][j], 0, 0, 0);
    // the next slab's way into LDS and the loads of the slab D after it
    fa.store(next, as_next);
    fb.store(next, bs_next);
    fa.load(next, s + 1 + D); fb.load(next, s + 1 + D);
    // order of issue: one matrix instruction, then in its shadow a share of the cutting (5 vector instructions) and
    // one LDS store; the four loads behind the last four matrix instructions
#pragma unroll
    for (int g = 0; g < 24; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
      __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
      if (g >= 20) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
  };
  // whole rounds of D slabs without a branch inside (a branch would make the wait before a stage's way into LDS
  // count every load in flight), then the rest
  int s0 = 0;
  for (; s0 + D <= nslab; s0 += D) {
#pragma unroll
    for (int d = 0; d < D; ++d) slab(s0 + d, d);
  }
#pragma unroll
  for (int d = 0; d < D - 1; ++d)
    if (s0 + d < nslab) slab(s0 + d, d);       // uniform over the workgroup

  store_tiles<2, 2>(p, kz, acc, m0 + wm * 64, n0 + wn * 64);
}

// The same for an operand that is already bf16 in memory (a copy written once, read by several products): half the
// bytes, no rounding in the loop.  KC: a unit is one 16-byte load of 8 consecutive k of a row and one 16-byte LDS
// store.  !KC: a unit is rows k and k + 1 of 8 columns (two 16-byte loads); each column's pair of k is one 32-bit
// LDS store, put together with a byte permute.  k and the contiguous dimension are multiples of 8 here.
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uintx4 buffer_load_u4(__amdgpu_buffer_rsrc_t rsrc, unsigned off) {
  return __builtin_bit_cast(uintx4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0));
}
template <int ROWS, bool KC>
struct SlabFeederB16 {
  // !KC: a pair of rows is loaded by one op and stored by two (columns 0..3, then 4..7), so that the LDS stores
  // spread over as many MFMA slots as those of the fp32 feeder
  static constexpr int kUnits = ROWS / 64;
  static constexpr int kLoads = KC ? ROWS / 64 : ROWS / 128;
  __amdgpu_buffer_rsrc_t rsrc;
  unsigned voff[kLoads][2];
  unsigned step;
  int lds_off[kLoads];
  int kq[kLoads];
  int klen;
  uintx4 r[kLoads][2];

  __device__ __forceinline__ void init(const unsigned short* ptr, int ld, int mn0, int MN, int kbeg, int kend) {
    const int tid = threadIdx.x;
    klen = kend - kbeg;
    if (KC) {
      const int rows = min(ROWS, MN - mn0);
      const unsigned short* base = ptr + (size_t)mn0 * ld + kbeg;
      rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned short*>(base), 0, (int)((size_t)rows * ld * 2 - (size_t)kbeg * 2), 0x00020000);
      step = BKH * 2;
#pragma unroll
      for (int u = 0; u < kLoads; ++u) {
        const int idx = tid + u * 256;
        const int row = idx >> 2, q = (idx & 3) * 8;
        voff[u][0] = (unsigned)row * (unsigned)ld * 2u + q * 2u;     // rows past the tile's last: beyond num_records
        voff[u][1] = 0;
        kq[u] = q;
        lds_off[u] = row * LDK + q;
      }
    } else {
      const unsigned short* base = ptr + (size_t)kbeg * ld + mn0;
      rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned short*>(base), 0, (int)((size_t)klen * ld * 2), 0x00020000);
      step = (unsigned)BKH * (unsigned)ld * 2u;
#pragma unroll
      for (int u = 0; u < kLoads; ++u) {
        const int idx = tid + u * 256;
        const int mn = (idx >> 4) * 8, k = (idx & 15) * 2;
#pragma unroll
        for (int h = 0; h < 2; ++h)
          voff[u][h] = (mn0 + mn < MN) ? (unsigned)(k + h) * (unsigned)ld * 2u + mn * 2u : kOutOfRange;
        kq[u] = 0;
        lds_off[u] = mn * LDK + k;
      }
    }
  }
  __device__ __forceinline__ void load(int u, int s) {
    if (KC) {
      const unsigned off = (s * BKH + kq[u] < klen) ? voff[u][0] + (unsigned)s * step : kOutOfRange;
      r[u][0] = buffer_load_u4(rsrc, off);
    } else if ((u & 1) == 0) {
      const int v = u >> 1;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const unsigned off = (s * BKH < klen) ? voff[v][h] + (unsigned)s * step : kOutOfRange;
        r[v][h] = buffer_load_u4(rsrc, off);
      }
    }
  }
  __device__ __forceinline__ void store(int u, unsigned short* slab) const {
    if (KC) {
      *reinterpret_cast<uintx4*>(slab + lds_off[u]) = r[u][0];
    } else {
      const int v = u >> 1, c0 = (u & 1) * 4;
      unsigned short* q = slab + lds_off[v];
#pragma unroll
      for (int c = c0; c < c0 + 4; ++c) {
        // column c of rows k (low half) and k + 1 (high half)
        const unsigned lo = r[v][0][c >> 1], hi = r[v][1][c >> 1];
        const unsigned w = (c & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        *reinterpret_cast<unsigned*>(q + c * LDK) = w;
      }
    }
  }
};

// M16: both operands are read as bf16 from memory (GemmP::A16, B16) instead of fp32 rounded on the way into LDS
template <int WM, int WN, bool TA, bool TB, bool M16>
__global__ __launch_bounds__(256) void gemm_mfma_bf16_v2_kernel(GemmP p) {
  constexpr int TMB = 64 * WM, TNB = 64 * WN;
  constexpr bool AKC = !TA, BKC = TB;
  extern __shared__ __align__(16) float smem[];
  unsigned short* As = reinterpret_cast<unsigned short*>(smem);     // [2][TMB][LDK]
  unsigned short* Bs = As + 2 * TMB * LDK;                          // [2][TNB][LDK]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  // A workgroup takes the items j = slot, slot + slots, ... of its XCD's range (see work_item): with a grid of
  // 8 * per_xcd workgroups that is one item each; with a grid of one workgroup per CU the workgroups stay and walk
  // through the items, and the stores of one tile drain while the next tile's slabs are already being fetched.
  const int slots = (int)(gridDim.x >> 3);
  for (int j = (int)(blockIdx.x >> 3); j < p.per_xcd; j += slots) {
  const int item = (int)(blockIdx.x & 7) * p.per_xcd + j;
  if (item >= p.work) break;
  const int kz = item / p.tiles;
  const int tile = item - kz * p.tiles;
  int tm, tn;
  tile_coords(p, tile, p.tiles / p.tiles_n, &tm, &tn);
  const int m0 = tm * TMB, n0 = tn * TNB;
  const int kbeg = kz * p.kchunk;
  const int kend = min(p.K, kbeg + p.kchunk);
  const int nslab = (kend - kbeg + BKH - 1) / BKH;

  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  using FeedA = typename std::conditional<M16, SlabFeederB16<TMB, AKC>, SlabFeederBf<TMB, AKC>>::type;
  using FeedB = typename std::conditional<M16, SlabFeederB16<TNB, BKC>, SlabFeederBf<TNB, BKC>>::type;
  FeedA fa;
  FeedB fb;
  if constexpr (M16) {
    fa.init(p.A16, p.lda, m0, p.M, kbeg, kend);
    fb.init(p.B16, p.ldb, n0, p.N, kbeg, kend);
  } else {
    fa.init(p.A, p.lda, m0, p.M, kbeg, kend);
    fb.init(p.B, p.ldb, n0, p.N, kbeg, kend);
  }
  constexpr int UA = FeedA::kUnits, UB = FeedB::kUnits;
  constexpr int NOPS = 2 * (UA + UB);            // stores of slab s+1 (A then B), then loads of slab s+2 (A then B)
  constexpr int NMFMA = 2 * WM * WN;             // per slab and wavefront
  constexpr int OPM = (NOPS + NMFMA - 1) / NMFMA;

#pragma unroll
  for (int u = 0; u < UA; ++u) fa.load(u, 0);
#pragma unroll
  for (int u = 0; u < UB; ++u) fb.load(u, 0);
#pragma unroll
  for (int u = 0; u < UA; ++u) fa.store(u, As);
#pragma unroll
  for (int u = 0; u < UB; ++u) fb.store(u, Bs);
#pragma unroll
  for (int u = 0; u < UA; ++u) fa.load(u, 1);
#pragma unroll
  for (int u = 0; u < UB; ++u) fb.load(u, 1);
  __syncthreads();

  for (int s = 0; s < nslab; ++s) {
    const int buf = s & 1;
    const unsigned short* as = As + buf * TMB * LDK + (wm * 32 * WM + l32) * LDK + lh * 8;
    const unsigned short* bs = Bs + buf * TNB * LDK + (wn * 32 * WN + l32) * LDK + lh * 8;
    unsigned short* as_next = As + (buf ^ 1) * TMB * LDK;
    unsigned short* bs_next = Bs + (buf ^ 1) * TNB * LDK;
#pragma unroll
    for (int ks = 0; ks < BKH; ks += 16) {
      bf16x8 af[WM], bfr[WN];
#pragma unroll
      for (int i = 0; i < WM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(as + i * 32 * LDK + ks);
#pragma unroll
      for (int j = 0; j < WN; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(bs + j * 32 * LDK + ks);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
          const int m = (ks / 16) * WM * WN + i * WN + j;       // index of this MFMA inside the slab
#pragma unroll
          for (int o = m * OPM; o < (m + 1) * OPM; ++o) {
            if (o < UA) fa.store(o, as_next);
            else if (o < UA + UB) fb.store(o - UA, bs_next);
            else if (o < 2 * UA + UB) fa.load(o - UA - UB, s + 2);
            else if (o < NOPS) fb.load(o - 2 * UA - UB, s + 2);
          }
          __builtin_amdgcn_sched_barrier(0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();
  }

  store_tiles<WM, WN>(p, kz, acc, m0 + wm * WM * 32, n0 + wn * WN * 32);
  }  // items of this workgroup
}

// ---------------------------------------------------------------------------
// The bf16-copy kernel for operands that are BOTH laid out along k (A16 [M,K], B16 stored [N,K]: the form every large
// product of the stack is brought into).  Same 256 x 256 tile, 2 x 2 wavefronts of 4 x 4 MFMA tiles and k slabs of 32
// as above; what differs is the way into LDS:
//  * buffer loads that write LDS directly (16 bytes per lane, lane i of a wavefront's load lands at the load's LDS base
//    + 16 i): no staging registers and no LDS store instructions, so a RING OF FOUR slabs fits (4 x 32 KB) and the
//    loads of slab s+3 are issued while slab s is multiplied - three slabs (1.3 us of matrix work) of lookahead
//    against one in the kernel above, whose staging registers hold no more and whose every slab waited for memory
//    (matrix cores busy 0.45 of the time with LDS only 0.25 busy; here 0.58).
//  * LDS rows are the slab's 32 k of one row, unpadded (64 bytes); the four 16-byte chunks of a row are permuted by
//    ring_swizzle(row), applied on the GLOBAL side of the load (the lane that fills chunk position c of a row fetches
//    chunk c ^ swizzle), so that the operand reads (one chunk of 8 or 16 neighbouring rows per group of lanes) touch
//    every bank once.
//  * operand fragments are read half a slab ahead of the MFMAs that use them; one barrier per slab, in its middle:
//      first half of slab s   MFMAs on f0 (k 0..15); beside them f1 (k 16..31) is read and slab s+3 is requested
//      wait for this wavefront's loads of slab s+1, barrier (every wavefront's have landed; everybody holds its f1,
//                             so the slab before s is free to be overwritten)
//      second half            MFMAs on f1; beside them f0 of slab s+1 is read
// Out-of-range lanes (rows past M or N, k past the slice) read zeros through the buffer resource's range check, which
// looks at the lane offset only: the slab's k offset is therefore added to the lane offset, not passed as the scalar
// offset.
constexpr int RING = 4;      // slabs in the ring (five, all 160 KB of LDS, measured no faster)
__device__ __forceinline__ int ring_swizzle(int row) { return (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1); }
typedef __attribute__((address_space(3))) void* lds_ptr_t;

__global__ __launch_bounds__(256) void gemm_bf16_ring_kernel(GemmP p) {
  constexpr int WM = 4, WN = 4, TMB = 256, TNB = 256;
  constexpr int OPB = TMB * BKH * 2;                                // bytes of one operand's slab (16 KB)
  extern __shared__ __align__(16) float smem[];
  unsigned char* ring = reinterpret_cast<unsigned char*>(smem);     // [RING][A slab | B slab]

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;
  const int swz = ring_swizzle(l32);                                // the lane's rows are l32 plus multiples of 32

  // this thread's four loads per operand and slab: load u of wavefront w fills LDS chunks [(4 u + w) 64, + 64)
  unsigned rowoff[4];      // row of the chunk inside the tile
  int klog[4];             // k offset (elements) of the chunk this lane fetches, inside a slab
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int pc = (u * 4 + wave) * 64 + lane;
    const int row = pc >> 2;
    rowoff[u] = (unsigned)row;
    klog[u] = ((pc & 3) ^ ring_swizzle(row)) * 8;
  }
  // LDS byte offsets of the lane's operand fragments inside a slab: row * 64 + permuted chunk * 16
  int fragoff[2][WM + WN];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int q = 0; q < WM + WN; ++q) {
      const int row = q < WM ? wm * 32 * WM + q * 32 + l32 : wn * 32 * WN + (q - WM) * 32 + l32;
      fragoff[h][q] = (q < WM ? 0 : OPB) + row * 64 + (((lh + 2 * h) ^ swz) << 4);
    }

  const int slots = (int)(gridDim.x >> 3);
  for (int j = (int)(blockIdx.x >> 3); j < p.per_xcd; j += slots) {
    const int item = (int)(blockIdx.x & 7) * p.per_xcd + j;
    if (item >= p.work) break;
    const int kz = item / p.tiles;
    const int tile = item - kz * p.tiles;
    int tm, tn;
    tile_coords(p, tile, p.tiles / p.tiles_n, &tm, &tn);
    const int m0 = tm * TMB, n0 = tn * TNB;
    const int kbeg = kz * p.kchunk;
    const int kend = min(p.K, kbeg + p.kchunk);
    const int klen = kend - kbeg;
    const int nslab = (klen + BKH - 1) / BKH;

    // rows past the tile's last valid one lie beyond num_records
    const int rowsA = min(TMB, p.M - m0), rowsB = min(TNB, p.N - n0);
    __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned short*>(p.A16 + (size_t)m0 * p.lda + kbeg), 0, (int)((size_t)rowsA * p.lda * 2 - (size_t)kbeg * 2), 0x00020000);
    __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned short*>(p.B16 + (size_t)n0 * p.ldb + kbeg), 0, (int)((size_t)rowsB * p.ldb * 2 - (size_t)kbeg * 2), 0x00020000);
    unsigned voffA[4], voffB[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      voffA[u] = rowoff[u] * (unsigned)p.lda * 2u + (unsigned)klog[u] * 2u;
      voffB[u] = rowoff[u] * (unsigned)p.ldb * 2u + (unsigned)klog[u] * 2u;
    }
    // load u (0..3: A, 4..7: B) of slab t into ring stage t % RING
    auto request = [&](int o, int t, int stage) {
      const int u = o & 3;
      const bool ink = t * BKH + klog[u] < klen;
      unsigned char* dst = ring + stage * 2 * OPB + (o < 4 ? 0 : OPB) + (u * 4 + wave) * 1024;
      const unsigned off = ink ? (o < 4 ? voffA[u] : voffB[u]) + (unsigned)t * (BKH * 2) : kOutOfRange;
      if (o < 4) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lds_ptr_t)dst, 16, (int)off, 0, 0, 0);
      else       __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB, (lds_ptr_t)dst, 16, (int)off, 0, 0, 0);
    };

    floatx16 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int jj = 0; jj < WN; ++jj)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][jj][r] = 0.f;

#pragma unroll
    for (int t = 0; t < RING - 1; ++t)
#pragma unroll
      for (int o = 0; o < 8; ++o) request(o, t, t);
    // 8 (RING - 1) loads in flight; the oldest 8 are slab 0
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(8 * (RING - 2)) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    bf16x8 f0[WM + WN], f1[WM + WN];
#pragma unroll
    for (int q = 0; q < WM + WN; ++q) f0[q] = *reinterpret_cast<const bf16x8*>(ring + fragoff[0][q]);

    int st_cur = 0;                                                 // ring stage of slab s
    for (int s = 0; s < nslab; ++s) {
      const int st_nxt = st_cur + 1 == RING ? 0 : st_cur + 1;
      const int st_req = st_cur == 0 ? RING - 1 : st_cur - 1;       // stage of slab s - 1 = of slab s + RING - 1
      const unsigned char* cur = ring + st_cur * 2 * OPB;
      const unsigned char* nxt = ring + st_nxt * 2 * OPB;
      // first half: f1 is read, then slab s + 3 is requested (its ring stage held slab s - 1, which nobody reads any more)
#pragma unroll
      for (int m = 0; m < WM * WN; ++m) {
        if (m < WM + WN) f1[m] = *reinterpret_cast<const bf16x8*>(cur + fragoff[1][m]);
        else request(m - (WM + WN), s + RING - 1, st_req);
        __builtin_amdgcn_sched_barrier(0);
        acc[m / WN][m % WN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0[m / WN], f0[WM + m % WN], acc[m / WN][m % WN], 0, 0, 0);
      }
      // slabs s+1 .. s+RING-1 are in flight (8 loads each): at most 8 (RING - 2) left means that slab s+1 has landed
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(8 * (RING - 2)) : "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      // (after the last slab this reads a stage that holds zeros or the next tile's first slab in the making: the
      // values are not used, the next tile reads its own f0 after its own barrier)
#pragma unroll
      for (int m = 0; m < WM * WN; ++m) {
        if (m < WM + WN) f0[m] = *reinterpret_cast<const bf16x8*>(nxt + fragoff[0][m]);
        __builtin_amdgcn_sched_barrier(0);
        acc[m / WN][m % WN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[m / WN], f1[WM + m % WN], acc[m / WN][m % WN], 0, 0, 0);
      }
      st_cur = st_nxt;
    }

    store_tiles<WM, WN>(p, kz, acc, m0 + wm * WM * 32, n0 + wn * WN * 32);
    // The next tile counts its own loads: nothing of this tile may be in flight (the requests past the last slab
    // returned zeros into ring stages; the stores above).  No barrier is needed: after the last slab's barrier no
    // wavefront reads LDS, and a wavefront's loads fill its own parts of the ring only.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
}

template <int WM, int WN, bool TA, bool TB, bool M16>
hipError_t launch_bf16_v2(hipStream_t stream, const GemmP& p, dim3 grid) {
  const size_t lds = (size_t)2 * 64 * (WM + WN) * LDK * sizeof(unsigned short);
  const void* fn = reinterpret_cast<const void*>(gemm_mfma_bf16_v2_kernel<WM, WN, TA, TB, M16>);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((gemm_mfma_bf16_v2_kernel<WM, WN, TA, TB, M16>), grid, dim3(256), lds, stream, p);
  return hipGetLastError();
}

template <typename K>
hipError_t launch_3xbf16_k(K kernel, hipStream_t stream, const GemmP& p, dim3 grid) {
  const size_t lds = gemm_3xbf16_lds_bytes();
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, grid, dim3(256), lds, stream, p);
  return hipGetLastError();
}
// buffer_loads: both operands made of whole, 16-byte aligned float4s and panels within 31-bit byte offsets.
// beside: the product shares its CUs with the recurrent kernels.  One slab in flight then: measured on the 4 x 500
// stack, two slabs in flight make the products a fifth faster and every recurrent step slower (54.1 against 52.8 ms
// per call), and the kernel keeps to 160 registers, which fit beside two wavefronts of any of the recurrent kernels that share CUs.
template <bool TA, bool TB>
hipError_t launch_3xbf16(hipStream_t stream, const GemmP& p, dim3 grid, bool vec, bool buffer_loads, bool beside) {
  if (buffer_loads && beside) return launch_3xbf16_k(gemm_f32_3xbf16_v2_kernel<TA, TB, 1>, stream, p, grid);
  if (buffer_loads) return launch_3xbf16_k(gemm_f32_3xbf16_v2_kernel<TA, TB, 2>, stream, p, grid);
  if (vec) return launch_3xbf16_k(gemm_f32_3xbf16_kernel<TA, TB, true>, stream, p, grid);
  return launch_3xbf16_k(gemm_f32_3xbf16_kernel<TA, TB, false>, stream, p, grid);
}

template <int WM, int WN, bool TA, bool TB, bool VEC>
hipError_t launch_bf16_v(hipStream_t stream, const GemmP& p, dim3 grid) {
  const size_t lds = (size_t)2 * 64 * (WM + WN) * LDK * sizeof(unsigned short);
  const void* fn = reinterpret_cast<const void*>(gemm_mfma_bf16_kernel<WM, WN, TA, TB, VEC>);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((gemm_mfma_bf16_kernel<WM, WN, TA, TB, VEC>), grid, dim3(256), lds, stream, p);
  return hipGetLastError();
}
template <bool TA, bool TB>
hipError_t launch_bf16(hipStream_t stream, const GemmP& p, dim3 grid, bool vec, bool big, bool pipelined, bool mem16, bool ring) {
  // the pipelined form pays with 256 x 256 tiles only (128 x 128: 204 against 294 TFLOP/s at 1000 x 4000 x 96000)
  if (pipelined && big && mem16 && !TA && TB && ring) {
    const size_t lds = (size_t)RING * 2 * 256 * BKH * 2;
    const void* fn = reinterpret_cast<const void*>(gemm_bf16_ring_kernel);
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gemm_bf16_ring_kernel, grid, dim3(256), lds, stream, p);
    return hipGetLastError();
  }
  if (pipelined && big && mem16) return launch_bf16_v2<4, 4, TA, TB, true>(stream, p, grid);
  if (pipelined && big) return launch_bf16_v2<4, 4, TA, TB, false>(stream, p, grid);
  if (big) return vec ? launch_bf16_v<4, 4, TA, TB, true>(stream, p, grid) : launch_bf16_v<4, 4, TA, TB, false>(stream, p, grid);
  return vec ? launch_bf16_v<2, 2, TA, TB, true>(stream, p, grid) : launch_bf16_v<2, 2, TA, TB, false>(stream, p, grid);
}

}  // namespace


namespace {
int current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); dev = 0; }
  return dev;
}
}  // namespace

hipError_t gemm(hipStream_t stream, const GemmCall& g) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  GemmP p;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.A = g.A; p.lda = g.lda; p.B = g.B; p.ldb = g.ldb; p.C = g.C; p.ldc = g.ldc;
  p.bias = g.bias; p.accumulate = g.accumulate ? 1 : 0;
  p.A16 = g.A16; p.B16 = g.B16;
  const bool bf16 = g.operand_dtype == 1;
  // bf16 operands: 256 x 256 tiles once those alone give every CU work
  // (or, where K is split into slices that multiply the work items, half as many such tiles)
  const long long big_tiles = (long long)((g.M + 255) / 256) * ((g.N + 255) / 256);
  const bool big = bf16 && !g.naive && !g.small_footprint &&
                   (big_tiles >= 128 || (g.splitk_ws && g.K >= 16 * 1024 && big_tiles >= 48));
  const int tile_m = big ? 256 : TM, tile_n = big ? 256 : TN;
  p.tiles_n = (g.N + tile_n - 1) / tile_n;
  p.band_m = p.tiles_n >= 8 ? 4 : 32 / p.tiles_n;
  p.kchunk = g.K; p.partial = nullptr;

  if (g.naive) {
    const size_t total = (size_t)g.M * g.N;
    hipLaunchKernelGGL(gemm_naive_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, p,
                       g.transA ? 1 : 0, g.transB ? 1 : 0, g.operand_dtype == 1 ? 1 : 0);
    return hipGetLastError();
  }

  // few columns on both sides and a long sum: the kernel with one tile for the whole of C
  if (!bf16 && g.transA && !g.transB && g.M <= 16 * TS_MB && g.N <= 16 * TS_NBW * TS_NW && g.K >= 16 * 1024 && g.splitk_ws &&
      !g.small_footprint && g.M % 4 == 0 && g.N % 4 == 0 && g.lda % 4 == 0 && g.ldb % 4 == 0 && aligned16(g.A) &&
      aligned16(g.B) && g.variant != 2) {
    const size_t per = (size_t)g.M * g.N;
    int slices = (int)std::min<size_t>(512, std::min<size_t>(g.splitk_floats / per, (size_t)g.K / (4 * TS_KC)));
    if (slices >= 2) {
      int kchunk = (g.K + slices - 1) / slices;
      kchunk = (kchunk + TS_KC - 1) / TS_KC * TS_KC;
      slices = (g.K + kchunk - 1) / kchunk;
      TsP t{g.A, g.B, g.splitk_ws, g.M, g.N, g.K, g.lda, g.ldb, kchunk};
      hipLaunchKernelGGL(tsmm_tn_f32_kernel, dim3((unsigned)slices), dim3(TS_THREADS), 0, stream, t);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      return splitk_reduce(stream, g.splitk_ws, slices, g.M, g.N, g.C, g.ldc, g.bias, g.accumulate);
    }
  }

  const int BK = bf16 ? BKH : 16;
  // float4 global loads need 16-byte aligned rows and whole float4s inside the matrix
  // (the dimension a float4 runs along must be a multiple of 4: k for an operand that is k-contiguous in
  // memory, m or n otherwise; the other dimension, and K of the weight-gradient products, may be anything)
  bool vec = aligned16(g.A) && aligned16(g.B) && (g.lda % 4 == 0) && (g.ldb % 4 == 0);
  vec = vec && ((g.transA ? g.M : g.K) % 4 == 0) && ((g.transB ? g.K : g.N) % 4 == 0);

  const int tiles_m = (g.M + tile_m - 1) / tile_m;
  const int tiles = tiles_m * p.tiles_n;
  int slices = 1;
  // K is split when the tiles alone leave CUs idle: always for long sums, and for sums of a few thousand when the
  // tiles do not even fill half the chip
  if (g.splitk_ws && tiles < 512 && (g.K >= 4 * 1024 || (g.K >= 1536 && tiles <= 160))) {
    // Alone: about 1024 work items (two workgroups per CU, two rounds).  Beside the recurrent kernels one workgroup
    // per CU fits, and every slice more is partial sums written and read through the memory path the recurrent
    // steps wait on: one work item per CU (the 4 x 500 stack: 52.4 -> 51.8 ms per call, backward steps beside the
    // weight gradients 7.23 -> 7.10 us; 384 items 52.4 ms, 128 items 55.9 ms).
    int items = 1024;
    if (g.small_footprint) {
      int cus = 0;
      if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, current_device()) != hipSuccess) { (void)hipGetLastError(); cus = 0; }
      items = cus > 0 ? cus : 256;
    }
    slices = (items + tiles - 1) / tiles;
    const int max_by_k = g.K / 512;
    if (slices > max_by_k) slices = max_by_k;
    const size_t per = (size_t)g.M * g.N;
    const size_t max_by_ws = g.splitk_floats / per;
    if ((size_t)slices > max_by_ws) slices = (int)max_by_ws;
    if (slices > 512) slices = 512;
    if (slices < 1) slices = 1;
  }
  if (slices > 1) {
    int kchunk = (g.K + slices - 1) / slices;
    kchunk = (kchunk + BK - 1) / BK * BK;
    slices = (g.K + kchunk - 1) / kchunk;
    p.kchunk = kchunk;
    p.partial = g.splitk_ws;
  }
  // the pipelined kernel addresses an operand panel with 31-bit byte offsets
  const size_t kspan = (size_t)p.kchunk;
  const size_t a_panel = g.transA ? kspan * g.lda * 4 : (size_t)tile_m * g.lda * 4;
  const size_t b_panel = g.transB ? (size_t)tile_n * g.ldb * 4 : kspan * g.ldb * 4;
  const bool pipelined_ok = a_panel < (1ull << 31) && b_panel < (1ull << 31);
  p.tiles = tiles;
  p.work = tiles * slices;
  p.per_xcd = (p.work + 7) / 8;
  dim3 grid((unsigned)(8 * p.per_xcd), 1, 1);
  hipError_t e;
  // variant 3 asks for the fp32 matrix instructions, chosen as variant 0 chose them before the three-part kernel;
  // it means nothing to bf16 operands
  const int variant = g.variant == 3 ? 0 : g.variant;
  const bool pipelined = vec && pipelined_ok && (variant == 1 || (variant == 0 && !g.small_footprint));
  if (bf16) {
    // bf16 copies of both operands are used where the kernel that takes them runs (256 x 256 tiles, pipelined) and
    // the copies consist of whole, 16-byte aligned groups of 8 values along their contiguous dimension
    const size_t a16_panel = g.transA16 ? kspan * g.lda16 * 2 : (size_t)tile_m * g.lda16 * 2;
    const size_t b16_panel = g.transB16 ? (size_t)tile_n * g.ldb16 * 2 : kspan * g.ldb16 * 2;
    const bool mem16 = g.A16 && g.B16 && big && (variant != 2) && aligned16(g.A16) && aligned16(g.B16) &&
                       g.lda16 % 8 == 0 && g.ldb16 % 8 == 0 && g.K % 8 == 0 && (g.transA16 ? g.M : g.K) % 8 == 0 &&
                       (g.transB16 ? g.K : g.N) % 8 == 0 && p.kchunk % 8 == 0 && a16_panel < (1ull << 31) && b16_panel < (1ull << 31);
    if (g.require_mem16 && !mem16) return hipErrorInvalidValue;
    bool tA = g.transA, tB = g.transB;
    if (mem16) { tA = g.transA16; tB = g.transB16; p.lda = g.lda16; p.ldb = g.ldb16; }
    const bool pl = mem16 || pipelined;
    if (mem16 && g.variant != kVariantNoWalk) {
      // one workgroup per CU (the kernel's LDS and registers allow no more), each walking through its XCD's items
      int cus = 0;
      if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, current_device()) != hipSuccess) { (void)hipGetLastError(); cus = 0; }
      const int slots = cus / 8;
      if (slots > 0 && slots < p.per_xcd) grid = dim3((unsigned)(8 * slots), 1, 1);
    }
    if (!tA && !tB)      e = launch_bf16<false, false>(stream, p, grid, vec, big, pl, mem16, g.variant != kVariantNoRing);
    else if (!tA && tB)  e = launch_bf16<false, true>(stream, p, grid, vec, big, pl, mem16, g.variant != kVariantNoRing);
    else if (tA && !tB)  e = launch_bf16<true, false>(stream, p, grid, vec, big, pl, mem16, g.variant != kVariantNoRing);
    else                 e = launch_bf16<true, true>(stream, p, grid, vec, big, pl, mem16, g.variant != kVariantNoRing);
  } else if (g.variant == 0) {
    // fp32 operands by default: the six-product form on the bf16 matrix cores (see gemm_f32_3xbf16_kernel)
    if (!g.transA && !g.transB)      e = launch_3xbf16<false, false>(stream, p, grid, vec, vec && pipelined_ok, g.small_footprint);
    else if (!g.transA && g.transB)  e = launch_3xbf16<false, true>(stream, p, grid, vec, vec && pipelined_ok, g.small_footprint);
    else if (g.transA && !g.transB)  e = launch_3xbf16<true, false>(stream, p, grid, vec, vec && pipelined_ok, g.small_footprint);
    else                             e = launch_3xbf16<true, true>(stream, p, grid, vec, vec && pipelined_ok, g.small_footprint);
  } else if (pipelined) {
    // A product that shares its CUs with the recurrent kernels keeps to the plain kernel: measured on the
    // 4 x 500 stack, the pipelined kernel beside them finishes its products sooner but slows every recurrent
    // step (6.04 / 9.37 us against 5.89 / 9.02 us), and the step chain is what bounds the pass.
    if (!g.transA && !g.transB)      e = launch_mfma_v2<false, false>(stream, p, grid);
    else if (!g.transA && g.transB)  e = launch_mfma_v2<false, true>(stream, p, grid);
    else if (g.transA && !g.transB)  e = launch_mfma_v2<true, false>(stream, p, grid);
    else                             e = launch_mfma_v2<true, true>(stream, p, grid);
  } else {
    // beside the recurrent kernels: the short matrix instruction (see gemm_mfma_f32_short_kernel); variant 2 keeps the long one
    const bool sh = g.small_footprint && variant != 2;
    if (!g.transA && !g.transB)      e = launch_mfma<16, false, false>(stream, p, grid, vec, sh);
    else if (!g.transA && g.transB)  e = launch_mfma<16, false, true>(stream, p, grid, vec, sh);
    else if (g.transA && !g.transB)  e = launch_mfma<16, true, false>(stream, p, grid, vec, sh);
    else                             e = launch_mfma<16, true, true>(stream, p, grid, vec, sh);
  }
  if (e != hipSuccess) return e;
  if (slices > 1) {
    e = splitk_reduce(stream, g.splitk_ws, slices, g.M, g.N, g.C, g.ldc, g.bias, g.accumulate);
  }
  return e;
}

namespace {
// fp32 -> bf16 (round to nearest even), 8 values per thread; n is a multiple of 8, both arrays 16-byte aligned
__global__ __launch_bounds__(256) void to_bf16_kernel(const float* __restrict__ src, unsigned short* __restrict__ dst, size_t n8) {
  const size_t gsz = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += gsz) {
    const float4 a = reinterpret_cast<const float4*>(src)[2 * i], b = reinterpret_cast<const float4*>(src)[2 * i + 1];
    uint4 w;
    w.x = pack_bf16(a.x, a.y); w.y = pack_bf16(a.z, a.w); w.z = pack_bf16(b.x, b.y); w.w = pack_bf16(b.z, b.w);
    reinterpret_cast<uint4*>(dst)[i] = w;
  }
}
}  // namespace

namespace {
// src [R, C] fp32 (row stride ld) -> dst [R, C] bf16 (row stride ldd; may be null) and dstT [C, R] bf16 (row stride R;
// may be null).  One workgroup per 128 x 128 tile; the transposed copy goes through LDS (as bf16) so that both are
// written in runs of 256 bytes per row.  R and C are multiples of 8.
constexpr int CV_T = 128;            // tile edge
constexpr int CV_LD = CV_T + 2;      // LDS row stride in bf16: an odd number of words, so a column walks the banks
__global__ __launch_bounds__(256) void to_bf16_2d_kernel(const float* __restrict__ src, int R, int C, int ld,
                                                          unsigned short* __restrict__ dst, int ldd, unsigned short* __restrict__ dstT) {
  __shared__ unsigned short tile[CV_T * CV_LD];
  const int tiles_c = (C + CV_T - 1) / CV_T;
  const int r0 = (int)(blockIdx.x / tiles_c) * CV_T, c0 = (int)(blockIdx.x % tiles_c) * CV_T;
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < CV_T * CV_T / 4 / 256; ++i) {
    const int idx = tid + i * 256;
    const int r = idx >> 5, c = (idx & 31) * 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    const bool in = r0 + r < R && c0 + c < C;
    if (in) v = *reinterpret_cast<const float4*>(src + (size_t)(r0 + r) * ld + c0 + c);
    uint2 w;
    w.x = pack_bf16(v.x, v.y); w.y = pack_bf16(v.z, v.w);
    if (dst && in) *reinterpret_cast<uint2*>(dst + (size_t)(r0 + r) * ldd + c0 + c) = w;
    if (dstT) {
      unsigned* q = reinterpret_cast<unsigned*>(tile + r * CV_LD + c);     // c and CV_LD are even: 4-byte aligned
      q[0] = w.x; q[1] = w.y;
    }
  }
  if (!dstT) return;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < CV_T * CV_T / 8 / 256; ++i) {
    const int idx = tid + i * 256;
    const int c = idx >> 4, r = (idx & 15) * 8;
    if (c0 + c < C && r0 + r < R) {
      unsigned short h[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) h[k] = tile[(r + k) * CV_LD + c];
      uint4 w;
      w.x = h[0] | ((unsigned)h[1] << 16); w.y = h[2] | ((unsigned)h[3] << 16);
      w.z = h[4] | ((unsigned)h[5] << 16); w.w = h[6] | ((unsigned)h[7] << 16);
      *reinterpret_cast<uint4*>(dstT + (size_t)(c0 + c) * R + r0 + r) = w;
    }
  }
}
}  // namespace

hipError_t to_bf16_2d(hipStream_t stream, const float* src, int R, int C, int ld, unsigned short* dst, int ldd, unsigned short* dstT) {
  if (ldd == 0) ldd = C;
  if (R % 8 != 0 || C % 8 != 0 || ld % 4 != 0 || ldd % 8 != 0 || ldd < C || !aligned16(src) || (dst && !aligned16(dst)) ||
      (dstT && !aligned16(dstT)))
    return hipErrorInvalidValue;
  if (R == 0 || C == 0) return hipSuccess;
  const size_t tiles = (size_t)((R + CV_T - 1) / CV_T) * ((C + CV_T - 1) / CV_T);
  hipLaunchKernelGGL(to_bf16_2d_kernel, dim3((unsigned)tiles), dim3(256), 0, stream, src, R, C, ld, dst, ldd, dstT);
  return hipGetLastError();
}

hipError_t to_bf16(hipStream_t stream, const float* src, unsigned short* dst, size_t n) {
  if (n % 8 != 0 || !aligned16(src) || !aligned16(dst)) return hipErrorInvalidValue;
  if (n == 0) return hipSuccess;
  const size_t n8 = n / 8;
  const unsigned grid = (unsigned)std::min<size_t>((n8 + 255) / 256, 16384);
  hipLaunchKernelGGL(to_bf16_kernel, dim3(grid), dim3(256), 0, stream, src, dst, n8);
  return hipGetLastError();
}

size_t gemm_small_lds_bytes(int operand_dtype, int variant) {
  if (operand_dtype == 1) return (size_t)2 * (TM + TN) * LDK * sizeof(unsigned short);
  return variant == 0 ? gemm_3xbf16_lds_bytes() : (size_t)4 * 16 * LDT * sizeof(float);
}

}  // namespace rlstm
