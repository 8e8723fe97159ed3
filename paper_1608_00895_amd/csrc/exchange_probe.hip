// Measurement aid (not part of the method): the bare per-step exchange that bounds the persistent
// recurrent kernels, without any of their arithmetic.  `groups` groups of `members` workgroups;
// per step every workgroup stores its tile with device-scope stores, waits for the
// acknowledgement, raises its step flag (64 copies, as the recurrent kernels do), polls the flags
// of all members of its group, then loads `read_bytes` of the group's tiles with device-scope
// 16-byte loads.  The time per step of this kernel is the floor of one hop of the recurrent
// kernels' step chain at the same group shape.  Same workgroup placement (index = member *
// groups + group), same bounded waits.
#include "rlstm_internal.h"

namespace rlstm {

namespace {

typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
constexpr int kCopies = 64, kCopyStride = 1024;
constexpr unsigned long long kWaitTicks = 100000000ull;   // 1 s of the 100 MHz wall clock

struct ProbeParams {
  unsigned* flags;      // [groups][kCopies][kCopyStride]
  unsigned* data;       // [groups][2][members * tile_bytes / 4]
  unsigned* err;
  unsigned long long* sink;
  int groups, members, tile_bytes, read_bytes, steps;
};

__global__ __launch_bounds__(256) void exchange_probe_kernel(ProbeParams p) {
  extern __shared__ char lds_pad[];              // only there to keep one workgroup per CU
  __shared__ int ok_lds;
  const int tid = threadIdx.x;
  const int grp = blockIdx.x % p.groups, wg = blockIdx.x / p.groups;
  if (p.steps < 0) lds_pad[tid] = 1;
  unsigned* flags = p.flags + (size_t)grp * kCopies * kCopyStride;
  const unsigned* myflags = flags + (size_t)(wg % kCopies) * kCopyStride;
  const size_t buf_words = (size_t)p.members * p.tile_bytes / 4;
  unsigned* base = p.data + (size_t)grp * 2 * buf_words;
  unsigned acc = 0;
  for (int s = 0; s < p.steps; ++s) {
    unsigned* cur = base + (size_t)(s & 1) * buf_words;
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(cur, 0, (int)(buf_words * 4), 0x00020000);
    const unsigned v = (unsigned)(s * 131 + wg);
    for (int i = tid * 16; i < p.tile_bytes; i += 256 * 16)
      __builtin_amdgcn_raw_buffer_store_b128(uintx4{v, v, v, v}, r, wg * p.tile_bytes + i, 0, 16);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid < kCopies)
      __hip_atomic_store(flags + (size_t)tid * kCopyStride + wg, (unsigned)(s + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid < 64) {
      int ok = 1;
      unsigned spins = 0;
      unsigned long long t0 = 0;
      for (;;) {
        bool all = true;
        for (int j = tid; j < p.members; j += 64)
          all = all && __hip_atomic_load(myflags + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= (unsigned)(s + 1);
        if (__all(all)) break;
        if ((++spins & 255u) == 0) {
          const unsigned long long now = wall_clock64();
          if (t0 == 0) t0 = now;
          else if (now - t0 > kWaitTicks) { ok = 0; break; }
          if (__hip_atomic_load(p.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) { ok = 0; break; }
        }
      }
      if (!ok) __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (tid == 0) ok_lds = ok;
    }
    __syncthreads();
    if (!ok_lds) break;
    // loads past the array's end return zero (buffer bounds)
    for (int i0 = 0; i0 < p.read_bytes; i0 += 256 * 16 * 8) {
      uintx4 w[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) w[q] = __builtin_amdgcn_raw_buffer_load_b128(r, i0 + (q * 256 + tid) * 16, 0, 16);
#pragma unroll
      for (int q = 0; q < 8; ++q) acc += w[q][0] ^ w[q][3];
    }
  }
  if (acc == 0xffffffffu) atomicAdd(p.sink, 1ull);   // keeps the loads alive
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

size_t exchange_probe_bytes(int groups, int members, int tile_bytes) {
  return 512 + (size_t)groups * kCopies * kCopyStride * 4 + align_up((size_t)groups * 2 * members * tile_bytes, 256);
}

hipError_t exchange_probe(hipStream_t stream, int groups, int members, int tile_bytes, int read_bytes, int steps,
                          void* ws, float* us_per_step, int* timed_out, int* resident_err) {
  DeviceInfo di;
  hipError_t e = device_info(&di);
  if (e != hipSuccess) return e;
  const size_t lds = di.max_lds / 2 + 1024;      // one workgroup per CU, like the recurrent kernels
  const void* fn = reinterpret_cast<const void*>(exchange_probe_kernel);
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  int per_cu = 0;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 256, lds);
  if (e != hipSuccess) return e;
  const int grid = groups * members;
  if ((long long)per_cu * di.num_cus < grid) { *resident_err = 1; return hipErrorCooperativeLaunchTooLarge; }
  char* w = static_cast<char*>(ws);
  ProbeParams p;
  p.err = reinterpret_cast<unsigned*>(w);
  p.sink = reinterpret_cast<unsigned long long*>(w + 256);
  p.flags = reinterpret_cast<unsigned*>(w + 512);
  p.data = p.flags + (size_t)groups * kCopies * kCopyStride;
  p.groups = groups; p.members = members; p.tile_bytes = tile_bytes; p.read_bytes = read_bytes; p.steps = steps;
  hipEvent_t e0, e1;
  e = hipEventCreate(&e0);
  if (e != hipSuccess) return e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) { (void)hipEventDestroy(e0); return e; }
  float best = 0.f;
  unsigned err_flag = 0;
  for (int rep = 0; rep < 3 && e == hipSuccess; ++rep) {
    e = hipMemsetAsync(ws, 0, exchange_probe_bytes(groups, members, tile_bytes), stream);
    if (e != hipSuccess) break;
    (void)hipEventRecord(e0, stream);
    void* args[] = {&p};
    e = hipLaunchKernel(fn, dim3((unsigned)grid), dim3(256), args, lds, stream);
    if (e != hipSuccess) break;
    (void)hipEventRecord(e1, stream);
    e = hipEventSynchronize(e1);
    if (e != hipSuccess) break;
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, e0, e1);
    if (e != hipSuccess) break;
    if (rep == 0 || ms < best) best = ms;
    unsigned f = 0;
    e = hipMemcpy(&f, p.err, sizeof(f), hipMemcpyDeviceToHost);
    err_flag |= f;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return e;
  *us_per_step = best * 1000.f / (float)steps;
  *timed_out = err_flag != 0 ? 1 : 0;
  return hipSuccess;
}

}  // namespace rlstm
