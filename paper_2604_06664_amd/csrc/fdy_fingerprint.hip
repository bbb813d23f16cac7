// fdy_fingerprint.hip - (b) topology fingerprint and template grouping for gfx950.
//
// Section 4.2.1 / Section 5.3: after capture a key is computed per graph over its structural
// properties; graphs with equal keys form one group that one template serves.  The key
// function (left open by the paper) is fixed in fdy.h: a SplitMix64-mixed hash per node,
// folded over the node sequence by Horner's rule H <- H*P + h_n.  Because
//     fold(a ++ b) = fold(a) * P^len(b) + fold(b)
// a segment is summarised by the pair (value, P^len) and segments combine associatively,
// so each graph is hashed by one workgroup as an ordered tree reduction and gives exactly
// the sequential 64-bit result.  Dense template ids in order of first appearance come from a
// hash table over the keys, built by the last block of the same launch to finish when the
// caller supplies a counter for that (fdy_segment_fingerprint with a prepared table), else by
// a second, single-workgroup launch; archives of more than 8,192 graphs use a table in the
// caller's workspace.
#include "fdy_device.hpp"
#include "fdy_internal.h"

namespace fdy {
namespace {

constexpr u64 kP = 0x9e3779b97f4a7c15ull;
// Threads per graph.  Measured on MI355X: 1,024 threads are more than graphs of a few hundred
// nodes can use; 256 are faster still for 576-node graphs (8.8 against 10.3 us for 67 of them)
// but slower for 2,632-node ones (13.5 against 11.5), and the host does not know the node
// counts.  512 is at least as fast as 1,024 on every shape tried.
constexpr int kFpBlock = 512;

__device__ __forceinline__ u64 mix(u64 x) {
  x ^= x >> 30;
  x *= 0xbf58476d1ce4e5b9ull;
  x ^= x >> 27;
  x *= 0x94d049bb133111ebull;
  x ^= x >> 31;
  return x;
}

__device__ __forceinline__ u64 node_hash(const fdy_node* n, u32 mask) {
  // 40-byte record read as five 8-byte words: kernel_id | grid.x,grid.y | grid.z,block.x |
  // block.y,block.z | blob_len,flags
  const u64* q = reinterpret_cast<const u64*>(n);
  u64 w0 = q[0], w1 = q[1], w2 = q[2], w3 = q[3], w4 = q[4];
  const u64 lo = 0x00000000ffffffffull, hi = 0xffffffff00000000ull;
  if (!(mask & FDY_FP_KERNEL_ID)) w0 = 0;
  w1 &= ((mask & FDY_FP_GRID_X) ? lo : 0) | ((mask & FDY_FP_GRID_Y) ? hi : 0);
  w2 &= ((mask & FDY_FP_GRID_Z) ? lo : 0) | ((mask & FDY_FP_BLOCK) ? hi : 0);
  if (!(mask & FDY_FP_BLOCK)) w3 = 0;
  w4 &= ((mask & FDY_FP_BLOB_LEN) ? lo : 0) | ((mask & FDY_FP_FLAGS) ? hi : 0);
  u64 a = mix(w0 + kP);
  a = mix(a ^ w1);
  a = mix(a ^ w2);
  a = mix(a ^ w3);
  a = mix(a ^ w4);
  return a;
}

// (v, p) summarises a segment: v = its Horner fold from 0, p = P^length.
struct Seg {
  u64 v, p;
};
__device__ __forceinline__ Seg combine(Seg left, Seg right) {
  return Seg{left.v * right.p + right.v, left.p * right.p};
}

// Grouping: template_id[g] = dense id, in order of first appearance, of g's key.  "First graph
// with the same key" comes from a hash table over the keys (open addressing, linear probing):
// a slot holds the lowest graph index seen so far of the one key that lives there.  A graph
// walks from its key's home slot until it meets an empty slot (and claims it) or its own key
// (and lowers the index there); slots are never emptied and every graph of a key walks the
// same way, so a key settles in exactly one slot.  O(G) expected, against the G^2 / 2
// comparisons of looking back at every earlier graph.
constexpr u32 kEmpty = 0xffffffffu;

__device__ __forceinline__ u32 home_slot(u64 key, u32 mask) { return (u32)(key >> 20) & mask; }  // keys are mixed already

template <typename KeyAt>
__device__ __forceinline__ void table_insert(u32* table, u32 mask, KeyAt key_at, u32 g) {
  const u64 k = key_at(g);
  u32 s = home_slot(k, mask);
  for (;;) {
    u32 cur = __hip_atomic_load(&table[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (cur == kEmpty) {
      const u32 old = atomicCAS(&table[s], kEmpty, g);
      if (old == kEmpty) return;
      cur = old;
    }
    if (key_at(cur) == k) {
      atomicMin(&table[s], g);
      return;
    }
    s = (s + 1) & mask;
  }
}

// After every graph has been inserted: the lowest graph index with g's key.
template <typename KeyAt>
__device__ __forceinline__ u32 table_first(const u32* table, u32 mask, KeyAt key_at, u32 g) {
  const u64 k = key_at(g);
  u32 s = home_slot(k, mask);
  for (;;) {
    const u32 cur = table[s];
    if (key_at(cur) == k) return cur;
    s = (s + 1) & mask;
  }
}

// Given first[g] in template_id[g]: ranks the firsts (chunked exclusive scan over the graphs, in
// order), writes tmpl_graph and replaces template_id by the dense ids.  One workgroup of T threads.
template <int T>
__device__ void rank_firsts(u32 G, u32* template_id, u32* tmpl_graph, u32* n_templates) {
  constexpr int kW = T / 64;
  __shared__ u32 s_w[kW + 1];
  __shared__ u32 s_carry;
  const u32 tid = threadIdx.x, l = lane_id(), w = tid >> 6;
  constexpr u32 kMark = 0x80000000u;
  if (tid == 0) s_carry = 0;
  __syncthreads();
  for (u32 g0 = 0; g0 < G; g0 += T) {
    const u32 g = g0 + tid;
    const bool first = g < G && template_id[g] == g;
    const u64 b = ballot(first);
    if (l == 0) s_w[w] = __popcll(b);
    __syncthreads();
    if (w == 0) {
      const u32 x = l < (u32)kW ? s_w[l] : 0;
      u32 xi = x;
#pragma unroll
      for (int d = 1; d < kW; d <<= 1) {
        const u32 o = __shfl_up(xi, d);
        if (l >= (u32)d) xi += o;
      }
      if (l < (u32)kW) s_w[l] = xi - x;
      if (l == (u32)kW - 1) s_w[kW] = xi;
    }
    __syncthreads();
    if (first) {
      const u32 rank = s_carry + s_w[w] + __popcll(b & lanemask_lt());
      template_id[g] = rank | kMark;
      if (tmpl_graph) tmpl_graph[rank] = g;
    }
    __syncthreads();
    if (tid == 0) s_carry += s_w[kW];
    __syncthreads();
  }
  // everyone else copies the rank of its first; then the marks come off
  for (u32 g = tid; g < G; g += T) {
    const u32 v = template_id[g];
    if (!(v & kMark)) template_id[g] = template_id[v] & ~kMark;
  }
  __syncthreads();
  for (u32 g = tid; g < G; g += T) {
    const u32 v = template_id[g];
    if (v & kMark) template_id[g] = v & ~kMark;
  }
  if (tid == 0) *n_templates = s_carry;
}

// Up to kSmallGraphs graphs: keys, firsts and ranks stay in LDS and registers, and the outputs
// are written once; the only round trips to memory are the load of the keys and the stores of
// the results.  (The general form below goes through template_id in memory between its steps,
// which is four more round trips: as long as everything else this launch does.)
constexpr u32 kSmallGraphs = 1024;
template <int T>
__device__ void group_small(const u64* keys, u32 G, u32* template_id, u32* tmpl_graph, u32* n_templates,
                            u32* table /* LDS, at least twice the graphs */) {
  constexpr int kW = T / 64, kPer = kSmallGraphs / T;
  __shared__ u64 s_keys[kSmallGraphs];
  __shared__ u32 s_rank[kSmallGraphs];
  __shared__ u32 s_cnt[kW + 1];
  const u32 tid = threadIdx.x, l = lane_id(), w = tid >> 6;
  u32 slots = 64;
  while (slots < 2 * G) slots <<= 1;
  const u32 mask = slots - 1;
  for (u32 i = tid; i < slots; i += T) table[i] = kEmpty;
#pragma unroll
  for (int c = 0; c < kPer; ++c) {
    const u32 g = (u32)c * T + tid;
    if (g < G) s_keys[g] = __hip_atomic_load(&keys[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  auto key_at = [&](u32 h) { return s_keys[h]; };
#pragma unroll
  for (int c = 0; c < kPer; ++c) {
    const u32 g = (u32)c * T + tid;
    if (g < G) table_insert(table, mask, key_at, g);
  }
  __syncthreads();
  u32 first[kPer];
#pragma unroll
  for (int c = 0; c < kPer; ++c) {
    const u32 g = (u32)c * T + tid;
    first[c] = g < G ? table_first(table, mask, key_at, g) : kEmpty;
  }
  u32 carry = 0;  // firsts in the chunks before this one (the same in every thread)
#pragma unroll
  for (int c = 0; c < kPer; ++c) {
    if ((u32)c * T >= G) break;  // uniform
    const u32 g = (u32)c * T + tid;
    const bool is_first = g < G && first[c] == g;
    const u64 b = ballot(is_first);
    if (l == 0) s_cnt[w] = __popcll(b);
    __syncthreads();
    if (w == 0) {
      const u32 x = l < (u32)kW ? s_cnt[l] : 0;
      u32 xi = x;
#pragma unroll
      for (int d = 1; d < kW; d <<= 1) {
        const u32 o = __shfl_up(xi, d);
        if (l >= (u32)d) xi += o;
      }
      if (l < (u32)kW) s_cnt[l] = xi - x;
      if (l == (u32)kW - 1) s_cnt[kW] = xi;
    }
    __syncthreads();
    if (is_first) {
      const u32 rank = carry + s_cnt[w] + __popcll(b & lanemask_lt());
      s_rank[g] = rank;
      if (tmpl_graph) tmpl_graph[rank] = g;
    }
    carry += s_cnt[kW];
    __syncthreads();
  }
#pragma unroll
  for (int c = 0; c < kPer; ++c) {
    const u32 g = (u32)c * T + tid;
    if (g < G) template_id[g] = s_rank[first[c]];
  }
  if (tid == 0) *n_templates = carry;
}

// The whole grouping by one workgroup of T threads, table in LDS: up to kLdsGraphs graphs.
constexpr u32 kLdsGraphs = 8192, kLdsSlots = 2 * kLdsGraphs;
template <int T>
__device__ void group_in_lds(const u64* keys, u32 G, u32* template_id, u32* tmpl_graph, u32* n_templates,
                             u32* table /* LDS, kLdsSlots */) {
  if (G <= kSmallGraphs) {
    group_small<T>(keys, G, template_id, tmpl_graph, n_templates, table);
    return;
  }
  const u32 tid = threadIdx.x;
  u32 slots = 64;  // at least twice the graphs
  while (slots < 2 * G) slots <<= 1;
  const u32 mask = slots - 1;
  for (u32 i = tid; i < slots; i += T) table[i] = kEmpty;
  __syncthreads();
  auto key_at = [&](u32 g) { return __hip_atomic_load(&keys[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
  for (u32 g = tid; g < G; g += T) table_insert(table, mask, key_at, g);
  __syncthreads();
  for (u32 g = tid; g < G; g += T) template_id[g] = table_first(table, mask, key_at, g);
  __syncthreads();
  rank_firsts<T>(G, template_id, tmpl_graph, n_templates);
}

struct FpArgs {
  const fdy_node* nodes;
  const u64* node_off;
  u32 mask;
  u64* keys;
  u32* template_id;
  u32* tmpl_graph;
  u32* n_templates;
  // relocation segmentation in the same launch (null relocs_off: none): block g answers
  // boundary g, the last block boundary G as well
  const fdy_reloc* relocs;
  const u64* d_count;
  u64 capacity;
  const u64* word_off;
  u64* reloc_off;
  // grouping in the same launch by the last block to finish (null: not here); the counter is
  // zero on entry and left zero
  u32* counter;
};

// One block per graph.  A launch of one block (an archive of a single graph) also writes the
// grouping: the graph is its own template.
__global__ __launch_bounds__(kFpBlock) void fp_key_kernel(FpArgs a) {
  __shared__ Seg s_seg[kFpBlock / 64];
  __shared__ u32 s_last;
  extern __shared__ __align__(16) u32 s_table[];  // grouping in this launch only
  const u32 g = blockIdx.x, tid = threadIdx.x, G = gridDim.x;
  const u64 n0 = a.node_off[g], N = a.node_off[g + 1] - n0;
  // contiguous chunk per thread, in thread order
  const u64 chunk = (N + kFpBlock - 1) / kFpBlock;
  u64 lo = (u64)tid * chunk, hi = lo + chunk;
  if (lo > N) lo = N;
  if (hi > N) hi = N;
  Seg s{0, 1};
  u64 i = lo;
  for (; i + 4 <= hi; i += 4) {  // four nodes' loads and mixes side by side, folded in order
    const u64 h0 = node_hash(a.nodes + n0 + i, a.mask), h1 = node_hash(a.nodes + n0 + i + 1, a.mask);
    const u64 h2 = node_hash(a.nodes + n0 + i + 2, a.mask), h3 = node_hash(a.nodes + n0 + i + 3, a.mask);
    s.v = (((s.v * kP + h0) * kP + h1) * kP + h2) * kP + h3;
    s.p *= kP * kP * kP * kP;
  }
  for (; i < hi; ++i) {
    s.v = s.v * kP + node_hash(a.nodes + n0 + i, a.mask);
    s.p *= kP;
  }
  // ordered reduction inside the wave: lane l absorbs lane l+d (its right neighbour block)
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    Seg r;
    r.v = __shfl_down(s.v, d);
    r.p = __shfl_down(s.p, d);
    if ((lane_id() & (2 * d - 1)) == 0) s = combine(s, r);
  }
  if (lane_id() == 0) s_seg[tid >> 6] = s;
  if (a.reloc_off) {
    // (a2) lower bound of this graph's first word among the relocation words, by the block's
    // last waves while the first one folds the partial hashes
    const u32 w = tid >> 6;
    const bool extra = g + 1 == G && w == kFpBlock / 64 - 2;  // boundary G: the end of the last graph
    if (w == kFpBlock / 64 - 1 || extra) {
      const u32 b = extra ? G : g;
      u64 n = *a.d_count;
      if (n > a.capacity) n = a.capacity;
      const fdy_reloc* relocs = a.relocs;
      const u64 target = a.word_off[b];
      // the first boundary is word 0 and the last lies behind every word: both are answered
      // without the search's dependent round trips
      u32 r = 0;
      if (target != 0 && n != 0)
        r = (u64)relocs[n - 1].word < target
                ? (u32)n
                : wave_lower_bound([&](u32 i) { return (u64)relocs[i].word; }, 0u, (u32)n, target);
      if (lane_id() == 0) a.reloc_off[b] = r;
    }
  }
  __syncthreads();
  if (tid == 0) {
    Seg t = s_seg[0];
    for (int w = 1; w < kFpBlock / 64; ++w) t = combine(t, s_seg[w]);
    const u64 key = mix(mix(N) * t.p + t.v);
    if (G == 1) {
      a.keys[g] = key;
      a.template_id[0] = 0;
      if (a.tmpl_graph) a.tmpl_graph[0] = 0;
      *a.n_templates = 1;
    } else if (a.counter) {
      // the key must have arrived (write-through, agent scope) before this block counts itself
      __hip_atomic_store(&a.keys[g], key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
      s_last = __hip_atomic_fetch_add(a.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == G;
    } else {
      a.keys[g] = key;
    }
  }
  if (G == 1 || !a.counter) return;
  __syncthreads();
  if (!s_last) return;
  if (tid == 0) __hip_atomic_store(a.counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  group_in_lds<kFpBlock>(a.keys, G, a.template_id, a.tmpl_graph, a.n_templates, s_table);
}

// Grouping as a launch of its own: one workgroup, table in LDS.
__global__ __launch_bounds__(1024) void fp_group_kernel(const u64* keys, u32 G, u32* template_id,
                                                        u32* tmpl_graph, u32* n_templates) {
  extern __shared__ __align__(16) u32 s_table[];
  group_in_lds<1024>(keys, G, template_id, tmpl_graph, n_templates, s_table);
}

// More graphs than the LDS table holds: the table lies in the caller's workspace and the steps
// are launches of their own (fill, insert, look up, rank).
__global__ void fp_table_fill_kernel(u32* table, u32 slots) {
  const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < slots) table[i] = kEmpty;
}
__global__ void fp_table_insert_kernel(const u64* keys, u32 G, u32* table, u32 mask) {
  const u32 g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g < G) table_insert(table, mask, [&](u32 h) { return keys[h]; }, g);
}
__global__ void fp_table_first_kernel(const u64* keys, u32 G, const u32* table, u32 mask, u32* template_id) {
  const u32 g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g < G) template_id[g] = table_first(table, mask, [&](u32 h) { return keys[h]; }, g);
}
__global__ __launch_bounds__(1024) void fp_rank_kernel(u32 G, u32* template_id, u32* tmpl_graph, u32* n_templates) {
  rank_firsts<1024>(G, template_id, tmpl_graph, n_templates);
}

u32 table_slots(u32 G) {
  u32 slots = 64;
  while (slots < 2 * (u64)G) slots <<= 1;
  return slots;
}

constexpr u32 kMaxGraphs = 1u << 20;

}  // namespace
}  // namespace fdy

using namespace fdy;

extern "C" size_t fdy_fingerprint_workspace_bytes(uint32_t n_graphs) {
  if (n_graphs > kMaxGraphs) return 0;
  return n_graphs > kLdsGraphs ? (size_t)table_slots(n_graphs) * 4 : 256;
}

static int fingerprint_launch(FpArgs a, uint32_t n_graphs, uint32_t n_boundaries, void* d_workspace,
                              size_t workspace_bytes, hipStream_t stream) {
  const bool big = n_graphs > kLdsGraphs;
  if (big && (!d_workspace || ((uintptr_t)d_workspace & 255) || workspace_bytes < (size_t)table_slots(n_graphs) * 4))
    return FDY_ERR_WORKSPACE;
  (void)hipGetLastError();  // drop any stale error left by earlier, unrelated runtime calls
  const size_t lds_table = big ? 0 : (size_t)table_slots(n_graphs) * 4;
  if (big) a.counter = nullptr;  // grouping by launches of its own
  if (n_graphs) {
    const size_t lds = a.counter && n_graphs > 1 ? lds_table : 0;
    if (lds > 32768)
      FDY_HIP_TRY(hipFuncSetAttribute((const void*)fp_key_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)(kLdsSlots * 4)));
    launch(FDY_PROF_FP_KEYS, fp_key_kernel, dim3(n_graphs), dim3(kFpBlock), lds, stream, a);
    FDY_HIP_TRY(hipGetLastError());
    if (n_graphs == 1 || a.counter) return FDY_OK;  // the key kernel has written the grouping too
  }
  if (!big) {
    if (lds_table > 32768)
      FDY_HIP_TRY(hipFuncSetAttribute((const void*)fp_group_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)(kLdsSlots * 4)));
    launch(FDY_PROF_FP_GROUP, fp_group_kernel, dim3(1), dim3(1024), lds_table, stream, (const u64*)a.keys, n_graphs,
           a.template_id, a.tmpl_graph, a.n_templates);
    FDY_HIP_TRY(hipGetLastError());
    return FDY_OK;
  }
  u32* table = (u32*)d_workspace;
  const u32 slots = table_slots(n_graphs), nb = (n_graphs + 255) / 256;
  prof_begin(FDY_PROF_FP_GROUP, stream);
  hipLaunchKernelGGL(fp_table_fill_kernel, dim3((slots + 255) / 256), dim3(256), 0, stream, table, slots);
  hipLaunchKernelGGL(fp_table_insert_kernel, dim3(nb), dim3(256), 0, stream, (const u64*)a.keys, n_graphs, table,
                     slots - 1);
  hipLaunchKernelGGL(fp_table_first_kernel, dim3(nb), dim3(256), 0, stream, (const u64*)a.keys, n_graphs,
                     (const u32*)table, slots - 1, a.template_id);
  hipLaunchKernelGGL(fp_rank_kernel, dim3(1), dim3(1024), 0, stream, n_graphs, a.template_id, a.tmpl_graph,
                     a.n_templates);
  prof_end(FDY_PROF_FP_GROUP, stream);
  FDY_HIP_TRY(hipGetLastError());
  return FDY_OK;
}

extern "C" int fdy_fingerprint(const fdy_node* d_nodes, const uint64_t* d_node_off, uint32_t n_graphs,
                               uint32_t field_mask, uint64_t* d_keys, uint32_t* d_template_id,
                               uint32_t* d_tmpl_graph, uint32_t* d_n_templates, void* d_workspace,
                               size_t workspace_bytes, void* hip_stream) {
  if (n_graphs > kMaxGraphs || (field_mask & ~FDY_FP_ALL)) return FDY_ERR_INVALID_ARG;
  if (!d_n_templates) return FDY_ERR_INVALID_ARG;
  if (n_graphs && (!d_node_off || !d_keys || !d_template_id)) return FDY_ERR_INVALID_ARG;
  if ((uintptr_t)d_nodes & 7) return FDY_ERR_INVALID_ARG;
  FpArgs a = FpArgs{};
  a.nodes = d_nodes;
  a.node_off = (const u64*)d_node_off;
  a.mask = field_mask;
  a.keys = (u64*)d_keys;
  a.template_id = d_template_id;
  a.tmpl_graph = d_tmpl_graph;
  a.n_templates = d_n_templates;
  return fingerprint_launch(a, n_graphs, 0, d_workspace, workspace_bytes, (hipStream_t)hip_stream);
}

extern "C" int fdy_segment_fingerprint(const fdy_reloc* d_relocs, const uint64_t* d_count, uint64_t reloc_capacity,
                                       const uint64_t* d_word_off, uint64_t* d_reloc_off,
                                       const fdy_node* d_nodes, const uint64_t* d_node_off, uint32_t n_graphs,
                                       uint32_t field_mask, uint64_t* d_keys, uint32_t* d_template_id,
                                       uint32_t* d_tmpl_graph, uint32_t* d_n_templates, void* d_prepared,
                                       void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (n_graphs > kMaxGraphs || (field_mask & ~FDY_FP_ALL)) return FDY_ERR_INVALID_ARG;
  if (!d_n_templates || !d_count || !d_word_off || !d_reloc_off) return FDY_ERR_INVALID_ARG;
  if (reloc_capacity && !d_relocs) return FDY_ERR_INVALID_ARG;
  if (n_graphs && (!d_node_off || !d_keys || !d_template_id)) return FDY_ERR_INVALID_ARG;
  if ((uintptr_t)d_nodes & 7 || (uintptr_t)d_prepared & 255) return FDY_ERR_INVALID_ARG;
  if (n_graphs == 0) {  // one boundary, no graph: the plain calls do it
    const int rc = fdy_reloc_segment(d_relocs, d_count, reloc_capacity, d_word_off, 1, d_reloc_off, hip_stream);
    if (rc != FDY_OK) return rc;
    return fdy_fingerprint(d_nodes, d_node_off, 0, field_mask, d_keys, d_template_id, d_tmpl_graph, d_n_templates,
                           d_workspace, workspace_bytes, hip_stream);
  }
  FpArgs a = FpArgs{};
  a.nodes = d_nodes;
  a.node_off = (const u64*)d_node_off;
  a.mask = field_mask;
  a.keys = (u64*)d_keys;
  a.template_id = d_template_id;
  a.tmpl_graph = d_tmpl_graph;
  a.n_templates = d_n_templates;
  a.relocs = d_relocs;
  a.d_count = (const u64*)d_count;
  a.capacity = reloc_capacity;
  a.word_off = (const u64*)d_word_off;
  a.reloc_off = (u64*)d_reloc_off;
  // the prepared table's header block holds a counter for this call (zero between calls)
  a.counter = d_prepared ? (u32*)((unsigned char*)d_prepared + 64) : nullptr;
  return fingerprint_launch(a, n_graphs, n_graphs + 1, d_workspace, workspace_bytes, (hipStream_t)hip_stream);
}
