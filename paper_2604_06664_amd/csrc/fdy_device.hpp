// Internal helpers shared by the HIP kernels of libfdy (gfx950, wave64).  Not installed.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "fdy.h"
#include "fdy_internal.h"

#define FDY_WAVE 64

#define FDY_HIP_TRY(expr)                      \
  do {                                         \
    hipError_t e__ = (expr);                   \
    if (e__ != hipSuccess) return FDY_ERR_HIP; \
  } while (0)

namespace fdy {

typedef uint64_t u64;
typedef uint32_t u32;

__device__ __forceinline__ u32 lane_id() { return __lane_id(); }

__device__ __forceinline__ u64 lanemask_lt() {
  const u32 l = lane_id();
  return l == 0 ? 0ull : (~0ull >> (64 - l));
}

__device__ __forceinline__ u64 ballot(bool p) { return __ballot(p); }

// 16-byte vector load / store of two 64-bit words
struct __attribute__((aligned(16))) u64x2 {
  u64 x, y;
};

__device__ __forceinline__ void raise_status(u32* d_status, u32 bit) {
  if (d_status) atomicOr(d_status, bit);
}

// Wave-cooperative lower bound.  key(i) must be non-decreasing over [lo, hi); every lane
// of the wave must call with the same arguments.  Returns the first index in [lo, hi] whose
// key is not below `target` (hi if none).  Each round probes 64 evenly spaced positions in
// parallel, so a range of n entries needs ceil(log64 n) dependent memory round trips
// instead of log2 n.
//
// The index space is 32-bit with hi <= 2^32 - 256 (every list this library searches is
// shorter), and the wave-uniform range is updated with 32-bit min/add only.  This is
// deliberate: hipcc 7.2 miscompiles a chain of two wave-uniform 64-bit compare+select
// steps for gfx950 (the second select reuses the first compare's SCC), which is exactly
// what a 64-bit version of this loop produces.
template <typename KeyFn>
__device__ __forceinline__ u32 wave_lower_bound(KeyFn key, u32 lo, u32 hi, u64 target) {
  const u32 l = lane_id();
  while (lo < hi) {
    const u32 n = hi - lo;
    const u32 stride = (n + 63u) >> 6;                 // ceil(n / 64) >= 1
    const u32 idx = lo + (l + 1u) * stride - 1u;       // this lane's probe, <= hi + 62
    u64 k = ~0ull;                                     // past the end: never below
    if (idx < hi) k = key(idx);
    const u32 c = (u32)__popcll(ballot(k < target));   // probes below the target (a prefix)
    // entries up to probe c-1 are below   => answer >= lo + c*stride
    // probe c, if it exists, is not below => answer <= lo + (c+1)*stride - 1
    const u32 nlo = min(lo + c * stride, hi);
    const u32 nhi = nlo + min(stride - 1u, hi - nlo);
    lo = nlo;
    hi = nhi;
  }
  return lo;
}

// Exclusive scan of one u64 per thread over a workgroup of whole waves (at most 1024 threads);
// returns the exclusive prefix and sets `total` (same in every thread).  s_buf: 17 u64 of LDS.
__device__ inline u64 block_excl_scan(u64 v, u64* s_buf, u64& total) {
  const u32 l = lane_id(), w = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  u64 inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const u64 o = __shfl_up(inc, d);
    if (l >= (u32)d) inc += o;
  }
  if (l == 63) s_buf[w] = inc;
  __syncthreads();
  if (w == 0) {
    const u64 x = l < n_waves ? s_buf[l] : 0;
    u64 xi = x;
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) {
      const u64 o = __shfl_up(xi, d);
      if (l >= (u32)d) xi += o;
    }
    if (l < 16) s_buf[l] = xi - x;
    if (l == 15) s_buf[16] = xi;
  }
  __syncthreads();
  const u64 r = s_buf[w] + inc - v;
  total = s_buf[16];
  __syncthreads();
  return r;
}

// One kernel launch on the caller's stream; when the bench has switched timing on for `slot`,
// the launch carries a pair of events that receive the kernel's own begin and end.
template <typename... KArgs, typename... Args>
inline void launch(int slot, void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                   Args&&... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
  void *a = nullptr, *b = nullptr;
  if (prof_take(slot, &a, &b))
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, stream, (hipEvent_t)a, (hipEvent_t)b, 0u,
                          static_cast<KArgs>(args)...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds, stream, static_cast<KArgs>(args)...);
}

}  // namespace fdy
