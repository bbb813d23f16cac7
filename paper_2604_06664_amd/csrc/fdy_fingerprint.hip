// fdy_fingerprint.hip - (b) topology fingerprint and template grouping for gfx950.
//
// Section 4.2.1 / Section 5.3: after capture a key is computed per graph over its structural
// properties; graphs with equal keys form one group that one template serves.  The key
// function (left open by the paper) is fixed in fdy.h: a SplitMix64-mixed hash per node,
// folded over the node sequence by Horner's rule H <- H*P + h_n.  Because
//     fold(a ++ b) = fold(a) * P^len(b) + fold(b)
// a segment is summarised by the pair (value, P^len) and segments combine associatively,
// so each graph is hashed by one workgroup as an ordered tree reduction and gives exactly
// the sequential 64-bit result.  A second, single-workgroup kernel turns keys into dense
// template ids in order of first appearance.
#include "fdy_device.hpp"
#include "fdy_tune.h"

namespace fdy {
namespace {

constexpr u64 kP = 0x9e3779b97f4a7c15ull;
constexpr int kFpBlock = 1024;

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

// A launch of one block (an archive of a single graph) also writes the grouping: the graph is
// its own template, and the grouping kernel's launch is saved.
__global__ __launch_bounds__(kFpBlock) void fp_key_kernel(const fdy_node* nodes, const u64* node_off,
                                                          u32 mask, u64* keys, u32* template_id,
                                                          u32* tmpl_graph, u32* n_templates) {
  __shared__ Seg s_seg[kFpBlock / 64];
  const u32 g = blockIdx.x, tid = threadIdx.x;
  const u64 n0 = node_off[g], N = node_off[g + 1] - n0;
  // contiguous chunk per thread, in thread order
  const u64 chunk = (N + kFpBlock - 1) / kFpBlock;
  u64 a = (u64)tid * chunk, b = a + chunk;
  if (a > N) a = N;
  if (b > N) b = N;
  Seg s{0, 1};
  for (u64 i = a; i < b; ++i) {
    s.v = s.v * kP + node_hash(nodes + n0 + i, mask);
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
  __syncthreads();
  if (tid == 0) {
    Seg t = s_seg[0];
    for (int w = 1; w < kFpBlock / 64; ++w) t = combine(t, s_seg[w]);
    keys[g] = mix(mix(N) * t.p + t.v);
    if (gridDim.x == 1) {
      template_id[0] = 0;
      if (tmpl_graph) tmpl_graph[0] = 0;
      *n_templates = 1;
    }
  }
}

// Dense ids in order of first appearance, in place in template_id (single workgroup).
__global__ __launch_bounds__(1024) void fp_group_kernel(const u64* keys, u32 G, u32* template_id,
                                                        u32* tmpl_graph, u32* n_templates) {
  __shared__ u32 s_w[17];
  __shared__ u32 s_carry;
  const u32 tid = threadIdx.x, l = lane_id(), w = tid >> 6;
  constexpr u32 kMark = 0x80000000u;
  // pass 1: first[g] = lowest h with the same key
  for (u32 g = tid; g < G; g += 1024) {
    const u64 k = keys[g];
    u32 f = g;
    for (u32 h = 0; h < g; ++h)
      if (keys[h] == k) {
        f = h;
        break;
      }
    template_id[g] = f;
  }
  if (tid == 0) s_carry = 0;
  __syncthreads();
  // pass 2: rank the firsts (chunked exclusive scan), mark them
  for (u32 g0 = 0; g0 < G; g0 += 1024) {
    const u32 g = g0 + tid;
    const bool first = g < G && template_id[g] == g;
    const u64 b = ballot(first);
    if (l == 0) s_w[w] = __popcll(b);
    __syncthreads();
    if (w == 0) {
      const u32 x = l < 16 ? s_w[l] : 0;
      u32 xi = x;
#pragma unroll
      for (int d = 1; d < 16; d <<= 1) {
        const u32 o = __shfl_up(xi, d);
        if (l >= (u32)d) xi += o;
      }
      if (l < 16) s_w[l] = xi - x;
      if (l == 15) s_w[16] = xi;
    }
    __syncthreads();
    if (first) {
      const u32 rank = s_carry + s_w[w] + __popcll(b & lanemask_lt());
      template_id[g] = rank | kMark;
      if (tmpl_graph) tmpl_graph[rank] = g;
    }
    __syncthreads();
    if (tid == 0) s_carry += s_w[16];
    __syncthreads();
  }
  // pass 3: everyone else copies the rank of its first; pass 4: strip the marks
  for (u32 g = tid; g < G; g += 1024) {
    const u32 v = template_id[g];
    if (!(v & kMark)) template_id[g] = template_id[v] & ~kMark;
  }
  __syncthreads();
  for (u32 g = tid; g < G; g += 1024) {
    const u32 v = template_id[g];
    if (v & kMark) template_id[g] = v & ~kMark;
  }
  if (tid == 0) *n_templates = s_carry;
}

}  // namespace
}  // namespace fdy

using namespace fdy;

extern "C" int fdy_fingerprint(const fdy_node* d_nodes, const uint64_t* d_node_off, uint32_t n_graphs,
                               uint32_t field_mask, uint64_t* d_keys, uint32_t* d_template_id,
                               uint32_t* d_tmpl_graph, uint32_t* d_n_templates, void* hip_stream) {
  if (n_graphs > 65536u || (field_mask & ~FDY_FP_ALL)) return FDY_ERR_INVALID_ARG;
  if (!d_n_templates) return FDY_ERR_INVALID_ARG;
  if (n_graphs && (!d_node_off || !d_keys || !d_template_id)) return FDY_ERR_INVALID_ARG;
  if ((uintptr_t)d_nodes & 7) return FDY_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)hip_stream;
  (void)hipGetLastError();  // drop any stale error left by earlier, unrelated runtime calls
  if (n_graphs) {
    prof_begin(FDY_PROF_FP_KEYS, stream);
    hipLaunchKernelGGL(fp_key_kernel, dim3(n_graphs), dim3(kFpBlock), 0, stream, d_nodes,
                       (const u64*)d_node_off, field_mask, (u64*)d_keys, d_template_id, d_tmpl_graph,
                       d_n_templates);
    prof_end(FDY_PROF_FP_KEYS, stream);
    FDY_HIP_TRY(hipGetLastError());
    if (n_graphs == 1) return FDY_OK;  // the key kernel has written the grouping too
  }
  prof_begin(FDY_PROF_FP_GROUP, stream);
  hipLaunchKernelGGL(fp_group_kernel, dim3(1), dim3(1024), 0, stream, (const u64*)d_keys, n_graphs,
                     d_template_id, d_tmpl_graph, d_n_templates);
  prof_end(FDY_PROF_FP_GROUP, stream);
  FDY_HIP_TRY(hipGetLastError());
  return FDY_OK;
}
