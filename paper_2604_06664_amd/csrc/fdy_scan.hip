// fdy_scan.hip - (a1) pointer scan and (a2) relocation segmentation for gfx950.
//
// The scan classifies every 8-byte word of the captured argument blobs against the sorted
// allocation table (the relaxation of Section 4.1.1's identical-layout requirement: find
// every embedded pointer kernel-agnostically, because argument buffers are opaque -
// Section 2.2, Appendix B).  It is a streaming pass bounded by HBM bandwidth:
//
//   * each workgroup draws tiles of TILE consecutive words from an atomic ticket, loads them
//     with 16-byte coalesced loads and rejects every word outside the table's span with one
//     subtract-and-compare;
//   * the surviving candidates are compacted (wave ballot + popcount ranks, one wave scans
//     the per-wave totals) into an LDS queue, so that the interval search runs on dense
//     lanes only;
//   * the search is hierarchical: a sampled level of the table (every 2^seg_log2-th base)
//     is staged in LDS once per workgroup and binary-searched there; the remaining steps run
//     on the table itself out of L2;
//   * hits are compacted a second time in word order; the tile's global output position
//     comes from a decoupled look-back over per-tile state words (flag and value packed in
//     one 64-bit word, agent-scope relaxed atomics), so the input is read exactly once and
//     the relocation table is written exactly once, in ascending word order.
//
// Tickets are handed out in increasing order and a workgroup only ever waits for tiles
// with smaller tickets, which are already running or finished; the wait is bounded by a
// spin limit after which FDY_ST_SPIN is raised and the kernel still terminates.
#include "fdy_device.hpp"
#include "fdy_tune.h"

namespace fdy {
namespace {

struct ScanParams {
  const u64* words;
  u64 n_words;
  const fdy_alloc* table;
  u32 n_alloc;
  fdy_reloc* relocs;
  u64 capacity;
  u64* d_count;
  u32* ticket;
  const u64* top;  // [top_n] sampled bases, padded with ~0
  u64* state;      // [n_tiles]
  u32 n_tiles;
  u32 top_n;     // power of two
  u32 seg_log2;  // table entries per sampled base = 1 << seg_log2
  u32* d_status;
  u32 spin_limit;
};

constexpr u64 kFlagAgg = 1ull << 62;
constexpr u64 kFlagInc = 2ull << 62;
constexpr u64 kValMask = (1ull << 62) - 1;

__device__ __forceinline__ u64 ld_state(const u64* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_state(u64* p, u64 v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ u32 wave_incl_scan_u32(u32 v) {
  const u32 l = lane_id();
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const u32 o = __shfl_up(v, d);
    if (l >= (u32)d) v += o;
  }
  return v;
}

__device__ __forceinline__ u64 wave_sum_u64(u64 v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

// Decoupled look-back, executed by one whole wave.  Returns the number of hits in all tiles
// before `tile` and publishes this tile's inclusive prefix.
__device__ u64 lookback(u64* state, u32 tile, u64 total, u32 spin_limit, u32* d_status) {
  const u32 l = lane_id();
  if (tile == 0) {
    if (l == 0) st_state(&state[0], kFlagInc | total);
    return 0;
  }
  if (l == 0) st_state(&state[tile], kFlagAgg | total);
  u64 excl = 0;
  long long pos = (long long)tile - 1;
  u32 spins = 0;
  for (;;) {
    const long long idx = pos - (long long)l;
    const u64 v = idx >= 0 ? ld_state(&state[idx]) : kFlagInc;  // before tile 0: prefix 0
    const u32 flag = (u32)(v >> 62);
    const u64 inc_mask = ballot(flag == 2);
    const u64 empty_mask = ballot(flag == 0);
    const u32 first_inc = inc_mask ? (u32)__ffsll((long long)inc_mask) - 1 : 64;
    const u64 need = first_inc >= 63 ? ~0ull : ((2ull << first_inc) - 1);  // lanes 0..first_inc
    if (empty_mask & need) {
      if (++spins > spin_limit) {  // bounded wait: give up, flag it, let successors proceed
        if (l == 0) raise_status(d_status, FDY_ST_SPIN);
        break;
      }
      __builtin_amdgcn_s_sleep(2);
      continue;
    }
    excl += wave_sum_u64(((need >> l) & 1) ? (v & kValMask) : 0);
    if (first_inc < 64) break;
    pos -= 64;
  }
  if (l == 0) st_state(&state[tile], kFlagInc | ((excl + total) & kValMask));
  return excl;
}

template <int BLOCK, int L>
__global__ __launch_bounds__(BLOCK) void scan_kernel(ScanParams p) {
  constexpr int NW = BLOCK / 64;
  constexpr int R = 2 * L;  // words per thread
  constexpr int TILE = BLOCK * R;
  static_assert(R * NW <= 64, "one wave scans the per-wave totals");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  u64* top = reinterpret_cast<u64*>(smem_raw);  // [top_n]
  u64* qw = top + p.top_n;                      // [TILE] candidate values
  u32* qi = reinterpret_cast<u32*>(qw + TILE);  // [TILE] candidate local word index
  __shared__ u32 s_tile, s_Q;
  __shared__ u32 s_wtot[64], s_htot[64];
  __shared__ u64 s_prefix;

  const u32 tid = threadIdx.x;
  const u32 lane = tid & 63;
  const u32 wave = tid >> 6;
  const u64 lt = lanemask_lt();

  for (u32 i = tid; i < p.top_n; i += BLOCK) top[i] = p.top[i];
  const u64 span_lo = p.table[0].base;
  const u64 span_len = p.table[p.n_alloc - 1].base + p.table[p.n_alloc - 1].size - span_lo;
  const u32 seg = 1u << p.seg_log2;

  for (;;) {
    if (tid == 0) s_tile = atomicAdd(p.ticket, 1u);
    __syncthreads();  // also orders the top[] fill before its first use
    const u32 tile = s_tile;
    if (tile >= p.n_tiles) break;
    const u64 wbase = (u64)tile * TILE;

    // ---- load + span pre-filter + candidate ranks
    u64 w[R];
    bool c[R];
    u32 crank[R];
    const bool full = wbase + TILE <= p.n_words;
#pragma unroll
    for (int k = 0; k < L; ++k) {
      const u64 idx = wbase + ((u64)k * BLOCK + tid) * 2;
      if (full) {
        const u64x2 v = *reinterpret_cast<const u64x2*>(p.words + idx);
        w[2 * k] = v.x;
        w[2 * k + 1] = v.y;
        c[2 * k] = (v.x - span_lo) < span_len;
        c[2 * k + 1] = (v.y - span_lo) < span_len;
      } else {
        const bool v0 = idx < p.n_words, v1 = idx + 1 < p.n_words;
        w[2 * k] = v0 ? p.words[idx] : 0;
        w[2 * k + 1] = v1 ? p.words[idx + 1] : 0;
        c[2 * k] = v0 && (w[2 * k] - span_lo) < span_len;
        c[2 * k + 1] = v1 && (w[2 * k + 1] - span_lo) < span_len;
      }
      const u64 b0 = ballot(c[2 * k]), b1 = ballot(c[2 * k + 1]);
      const u32 pre = __popcll(b0 & lt) + __popcll(b1 & lt);
      crank[2 * k] = pre;
      crank[2 * k + 1] = pre + (c[2 * k] ? 1u : 0u);
      if (lane == 0) s_wtot[k * NW + wave] = __popcll(b0) + __popcll(b1);
    }
    __syncthreads();
    if (wave == 0) {
      const u32 v = lane < L * NW ? s_wtot[lane] : 0;
      const u32 inc = wave_incl_scan_u32(v);
      if (lane < L * NW) s_wtot[lane] = inc - v;
      if (lane == 63) s_Q = inc;
    }
    __syncthreads();
    const u32 Q = s_Q;
#pragma unroll
    for (int k = 0; k < L; ++k) {
      const u32 base = s_wtot[k * NW + wave];
      const u32 li = (k * BLOCK + tid) * 2;
      if (c[2 * k]) {
        qw[base + crank[2 * k]] = w[2 * k];
        qi[base + crank[2 * k]] = li;
      }
      if (c[2 * k + 1]) {
        qw[base + crank[2 * k + 1]] = w[2 * k + 1];
        qi[base + crank[2 * k + 1]] = li + 1;
      }
    }
    __syncthreads();

    // ---- interval search on the dense candidate queue
    bool hit[R];
    u32 hreg[R], hidx[R], hrank[R];
    u64 hoff[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      hit[r] = false;
      hreg[r] = 0;
      hidx[r] = 0;
      hoff[r] = 0;
      hrank[r] = 0;
      if ((u32)r * BLOCK < Q) {  // uniform over the workgroup
        const u32 q = r * BLOCK + tid;
        if (q < Q) {
          const u64 wv = qw[q];
          u32 i = 0;
          for (u32 step = p.top_n >> 1; step; step >>= 1)
            if (top[i + step] <= wv) i += step;
          u64 j = (u64)i << p.seg_log2;
          for (u32 step = seg >> 1; step; step >>= 1) {
            const u64 jj = j + step;
            if (jj < p.n_alloc && p.table[jj].base <= wv) j = jj;
          }
          const u64x2 e = *reinterpret_cast<const u64x2*>(&p.table[j]);
          hoff[r] = wv - e.x;
          hreg[r] = (u32)j;
          hidx[r] = qi[q];
          hit[r] = hoff[r] < e.y;
        }
        const u64 b = ballot(hit[r]);
        hrank[r] = __popcll(b & lt);
        if (lane == 0) s_htot[r * NW + wave] = __popcll(b);
      } else if (lane == 0) {
        s_htot[r * NW + wave] = 0;
      }
    }
    __syncthreads();
    if (wave == 0) {
      const u32 v = lane < R * NW ? s_htot[lane] : 0;
      const u32 inc = wave_incl_scan_u32(v);
      if (lane < R * NW) s_htot[lane] = inc - v;
      const u32 H = __shfl(inc, 63);
      const u64 excl = lookback(p.state, tile, H, p.spin_limit, p.d_status);
      if (lane == 0) {
        s_prefix = excl;
        if (tile == p.n_tiles - 1) {
          *p.d_count = excl + H;
          if (excl + H > p.capacity) raise_status(p.d_status, FDY_ST_CAPACITY);
        }
      }
    }
    __syncthreads();
    const u64 prefix = s_prefix;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (hit[r]) {
        const u64 pos = prefix + s_htot[r * NW + wave] + hrank[r];
        if (pos < p.capacity) {
          fdy_reloc o;
          o.word = (u32)(wbase + hidx[r]);
          o.region = hreg[r];
          o.offset = hoff[r];
          *reinterpret_cast<uint4*>(&p.relocs[pos]) = *reinterpret_cast<const uint4*>(&o);
        }
      }
    }
    // the barrier at the top of the next iteration separates these reads of s_htot /
    // s_prefix and the queue from the next tile's writes
  }
}

// Builds the sampled top level, clears the tile states and the ticket.
__global__ void scan_init_kernel(const fdy_alloc* table, u32 n_alloc, u64* top, u32 top_n,
                                 u32 seg_log2, u64* state, u32 n_tiles, u32* ticket, u64* d_count) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < top_n) {
    const u64 j = i << seg_log2;
    top[i] = j < n_alloc ? table[j].base : ~0ull;
  }
  if (i < n_tiles) state[i] = 0;
  if (i == 0) {
    *ticket = 0;
    if (n_tiles == 0 || n_alloc == 0) *d_count = 0;
  }
}

// (a2) one wave per boundary: lower bound of word_off[s] among the reloc words.
__global__ void reloc_segment_kernel(const fdy_reloc* relocs, const u64* d_count, u64 capacity,
                                     const u64* word_off, u32 n_off, u64* reloc_off) {
  const u32 s = blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6);
  if (s >= n_off) return;
  u64 n = *d_count;
  if (n > capacity) n = capacity;
  const u64 target = word_off[s];
  const u32 r = wave_lower_bound([&](u32 i) { return (u64)relocs[i].word; }, 0u, (u32)n, target);
  if (lane_id() == 0) reloc_off[s] = r;
}

constexpr u64 kMaxWords = (1ull << 32) - 256;  // word and reloc indices are 32-bit
constexpr int kBlock = 512;
constexpr int kL = 2;
constexpr int kTile = kBlock * kL * 2;

u32 pow2_ceil(u32 v) {
  u32 p = 1;
  while (p < v) p <<= 1;
  return p;
}

struct ScanPlan {
  u32 top_n, seg_log2, n_tiles;
  size_t off_top, off_state, total;
};

ScanPlan make_plan(u64 n_words, u32 n_alloc) {
  ScanPlan pl;
  const u32 top_cap = 1u << fdy__tune_get(FDY_TUNE_SCAN_TOP_LOG2);
  u32 seg_log2 = 0;
  while ((((u64)n_alloc + (1ull << seg_log2) - 1) >> seg_log2) > top_cap) ++seg_log2;
  const u32 sampled = (u32)(((u64)n_alloc + (1ull << seg_log2) - 1) >> seg_log2);
  pl.top_n = pow2_ceil(sampled < 2 ? 2 : sampled);
  pl.seg_log2 = seg_log2;
  pl.n_tiles = (u32)((n_words + kTile - 1) / kTile);
  pl.off_top = 256;
  pl.off_state = pl.off_top + (((size_t)pl.top_n * 8 + 255) & ~(size_t)255);
  pl.total = pl.off_state + (((size_t)pl.n_tiles * 8 + 255) & ~(size_t)255);
  return pl;
}

}  // namespace
}  // namespace fdy

using namespace fdy;

extern "C" size_t fdy_scan_workspace_bytes(uint64_t n_words, uint32_t n_alloc) {
  if (n_words > kMaxWords) return 0;
  return make_plan(n_words, n_alloc).total;
}

extern "C" int fdy_scan_pointers(const uint64_t* d_words, uint64_t n_words, const fdy_alloc* d_table,
                                 uint32_t n_alloc, fdy_reloc* d_relocs, uint64_t reloc_capacity,
                                 uint64_t* d_count, void* d_workspace, size_t workspace_bytes,
                                 uint32_t* d_status, void* hip_stream) {
  if (n_words > kMaxWords) return FDY_ERR_INVALID_ARG;
  if (!d_count) return FDY_ERR_INVALID_ARG;
  if (n_words && (!d_words || ((uintptr_t)d_words & 15))) return FDY_ERR_INVALID_ARG;
  if (n_alloc && (!d_table || ((uintptr_t)d_table & 15))) return FDY_ERR_INVALID_ARG;
  if (reloc_capacity && (!d_relocs || ((uintptr_t)d_relocs & 15))) return FDY_ERR_INVALID_ARG;
  const ScanPlan pl = make_plan(n_words, n_alloc);
  if (!d_workspace || ((uintptr_t)d_workspace & 255) || workspace_bytes < pl.total)
    return FDY_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)hip_stream;
  (void)hipGetLastError();  // drop any stale error left by earlier, unrelated runtime calls
  unsigned char* ws = (unsigned char*)d_workspace;
  u32* ticket = (u32*)ws;
  u64* top = (u64*)(ws + pl.off_top);
  u64* state = (u64*)(ws + pl.off_state);

  const u32 n_init = pl.top_n > pl.n_tiles ? pl.top_n : pl.n_tiles;
  prof_begin(FDY_PROF_SCAN_INIT, stream);
  hipLaunchKernelGGL(scan_init_kernel, dim3((n_init + 255) / 256), dim3(256), 0, stream,
                     d_table, n_alloc, top, pl.top_n, pl.seg_log2, state, pl.n_tiles, ticket,
                     (u64*)d_count);
  prof_end(FDY_PROF_SCAN_INIT, stream);
  FDY_HIP_TRY(hipGetLastError());
  if (pl.n_tiles == 0 || n_alloc == 0) return FDY_OK;  // nothing can be a pointer

  ScanParams p;
  p.words = (const u64*)d_words;
  p.n_words = n_words;
  p.table = d_table;
  p.n_alloc = n_alloc;
  p.relocs = d_relocs;
  p.capacity = reloc_capacity;
  p.d_count = (u64*)d_count;
  p.ticket = ticket;
  p.top = top;
  p.state = state;
  p.n_tiles = pl.n_tiles;
  p.top_n = pl.top_n;
  p.seg_log2 = pl.seg_log2;
  p.d_status = d_status;
  p.spin_limit = (u32)fdy__tune_get(FDY_TUNE_SCAN_SPIN_LIMIT);

  const size_t lds = (size_t)pl.top_n * 8 + (size_t)kTile * 12;
  int dev = 0, n_cu = 256;
  FDY_HIP_TRY(hipGetDevice(&dev));
  FDY_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  auto kern = scan_kernel<kBlock, kL>;
  FDY_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds));
  const u32 per_cu = (u32)fdy__tune_get(FDY_TUNE_SCAN_WG_PER_CU);
  u32 grid = (u32)n_cu * per_cu;
  if (grid > pl.n_tiles) grid = pl.n_tiles;
  prof_begin(FDY_PROF_SCAN_MAIN, stream);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), lds, stream, p);
  prof_end(FDY_PROF_SCAN_MAIN, stream);
  FDY_HIP_TRY(hipGetLastError());
  return FDY_OK;
}

extern "C" int fdy_reloc_segment(const fdy_reloc* d_relocs, const uint64_t* d_count,
                                 uint64_t reloc_capacity, const uint64_t* d_word_off, uint32_t n_off,
                                 uint64_t* d_reloc_off, void* hip_stream) {
  if (n_off == 0) return FDY_OK;
  if (!d_count || !d_word_off || !d_reloc_off) return FDY_ERR_INVALID_ARG;
  if (reloc_capacity && !d_relocs) return FDY_ERR_INVALID_ARG;
  (void)hipGetLastError();
  prof_begin(FDY_PROF_SEGMENT, hip_stream);
  hipLaunchKernelGGL(reloc_segment_kernel, dim3((n_off + 3) / 4), dim3(256), 0,
                     (hipStream_t)hip_stream, d_relocs, (const u64*)d_count, reloc_capacity,
                     (const u64*)d_word_off, n_off, (u64*)d_reloc_off);
  prof_end(FDY_PROF_SEGMENT, hip_stream);
  FDY_HIP_TRY(hipGetLastError());
  return FDY_OK;
}
