// fdy_derive.hip - override derivation for gfx950: the SAVE side of templating.
//
// Section 4.2.1 / Section 5.3: graphs of one topology group "differ only in per-node
// parameters", so a non-template graph is stored as what differs from its template.  For
// graph g with template source graph s, every 32-bit half of g's argument words that is not
// equal to s's half at the same place becomes an fdy_ovr32 {byte offset, value}, ascending
// per graph, graphs in order: exactly the override lists fdy_materialize consumes.
//
//   prep  (one workgroup)    checks each graph against its template (index, word count) and
//                            prefix-sums the graphs' tile counts (2048 words per tile);
//   count (tile)             compares the tile with the template's, counts differing halves;
//   scan  (one workgroup)    exclusive prefix over the tile counts -> each tile's output
//                            position, each graph's offset, the total;
//   write (tile)             compares again and writes the entries in order.
// The archive is read twice (it is small next to what materialize writes from it: one
// template and a list of scalars per graph); ordering inside a tile comes from ballots over
// words in index order, low half before high half.
#include "fdy_device.hpp"
#include "fdy_internal.h"

namespace fdy {
namespace {

constexpr int kDerTile = 2048;  // words per tile
constexpr int kDerBlock = 256;
constexpr int kDerRounds = kDerTile / kDerBlock;  // words per thread

struct DerWs {
  u64* tile_off;   // [G+1] first tile of each graph
  u32* tile_cnt;   // [max_tiles]
  u64* tile_pos;   // [max_tiles] entries before the tile
  u32* n_tiles;    // tiles in use
  u32 max_tiles;
};

struct DerParams {
  const u64* words;
  const u64* word_off;
  u32 n_graphs;
  const u32* graph_tmpl;
  const u32* tmpl_graph;
  u32 n_templates;
  u64 n_words_total;
  fdy_ovr32* ovr;
  u64 capacity;
  u64* ovr_off;
  u32* d_status;
  DerWs ws;
};

// Words of graph g that take part: 0 for a graph that cannot be compared (flagged).
__device__ __forceinline__ u64 comparable_words(const DerParams& p, u32 g, u32* src, bool* bad_index,
                                                bool* bad_size) {
  const u32 t = p.graph_tmpl[g];
  const u32 s = t < p.n_templates ? p.tmpl_graph[t] : 0xffffffffu;
  *src = s;
  if (s >= p.n_graphs) {
    *bad_index = true;
    return 0;
  }
  const u64 nw = p.word_off[g + 1] - p.word_off[g];
  if (p.word_off[s + 1] - p.word_off[s] != nw || (nw >> 29)) {  // byte offsets are 32-bit
    *bad_size = true;
    return 0;
  }
  return nw;
}

__global__ __launch_bounds__(1024) void derive_prep_kernel(DerParams p) {
  __shared__ u64 s_buf[17];
  const u32 G = p.n_graphs;
  u64 carry = 0;
  bool bad_index = false, bad_size = false;
  for (u32 g0 = 0; g0 < G; g0 += 1024) {
    const u32 g = g0 + threadIdx.x;
    u64 nt = 0;
    if (g < G) {
      u32 s;
      const u64 nw = comparable_words(p, g, &s, &bad_index, &bad_size);
      nt = (nw + kDerTile - 1) / kDerTile;
    }
    u64 total;
    const u64 e = block_excl_scan(nt, s_buf, total);
    if (g < G) p.ws.tile_off[g] = carry + e;
    carry += total;
  }
  if (bad_index) raise_status(p.d_status, FDY_ST_BAD_INDEX);
  if (bad_size) raise_status(p.d_status, FDY_ST_BAD_SIZE);
  if (threadIdx.x == 0) {
    const bool ok = p.word_off[G] == p.n_words_total && carry <= p.ws.max_tiles;
    if (!ok) raise_status(p.d_status, FDY_ST_BAD_SIZE);
    p.ws.tile_off[G] = ok ? carry : 0;
    *p.ws.n_tiles = ok ? (u32)carry : 0u;
  }
}

// kWrite = false: count the tile's differing halves; true: write them from tile_pos.
template <bool kWrite>
__global__ __launch_bounds__(kDerBlock) void derive_tile_kernel(DerParams p) {
  __shared__ u32 s_cnt[kDerRounds][kDerBlock / 64];
  const u32 j = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (j >= *p.ws.n_tiles) return;
  // largest g with tile_off[g] <= j
  u32 lo = 0, hi = p.n_graphs;  // answer in [lo, hi)
  while (hi - lo > 1) {
    const u32 mid = lo + (hi - lo) / 2;
    if (p.ws.tile_off[mid] <= j) lo = mid;
    else hi = mid;
  }
  const u32 g = lo;
  const u32 s = p.tmpl_graph[p.graph_tmpl[g]];  // valid: a graph that failed the checks has no tiles
  const u64 nw = p.word_off[g + 1] - p.word_off[g];
  const u64 k0 = ((u64)j - p.ws.tile_off[g]) * kDerTile;
  const u32 n = (u32)(nw - k0 < (u64)kDerTile ? nw - k0 : (u64)kDerTile);
  const u64* a = p.words + p.word_off[g] + k0;
  const u64* b = p.words + p.word_off[s] + k0;
  const u64 lt = lanemask_lt();
  // words in index order: round i covers words [256 i, 256 i + 256), one per thread
  u64 va[kDerRounds];
  bool dlo[kDerRounds], dhi[kDerRounds];
  u32 rank[kDerRounds];
#pragma unroll
  for (int i = 0; i < kDerRounds; ++i) {
    const u32 k = (u32)i * kDerBlock + tid;
    va[i] = 0;
    u64 vb = 0;
    if (k < n) {
      va[i] = a[k];
      vb = b[k];
    }
    const u64 x = va[i] ^ vb;
    dlo[i] = (u32)x != 0;
    dhi[i] = (u32)(x >> 32) != 0;
    const u64 blo = ballot(dlo[i]), bhi = ballot(dhi[i]);
    rank[i] = __popcll(blo & lt) + __popcll(bhi & lt);
    if (lane == 0) s_cnt[i][wave] = __popcll(blo) + __popcll(bhi);
  }
  __syncthreads();
  if (!kWrite) {
    if (tid == 0) {
      u32 c = 0;
      for (int i = 0; i < kDerRounds; ++i)
        for (int w = 0; w < kDerBlock / 64; ++w) c += s_cnt[i][w];
      p.ws.tile_cnt[j] = c;
    }
    return;
  }
  const u64 pos0 = p.ws.tile_pos[j];
  u32 before = 0;  // entries of the tile before this wave's share of round i
#pragma unroll
  for (int i = 0; i < kDerRounds; ++i) {
    u32 mine = before;
    for (u32 w = 0; w < wave; ++w) mine += s_cnt[i][w];
    const u32 byte_off = (u32)((k0 + (u64)i * kDerBlock + tid) * 8);
    u64 at = pos0 + mine + rank[i];
    if (dlo[i]) {
      if (at < p.capacity) p.ovr[at] = fdy_ovr32{byte_off, (u32)va[i]};
      ++at;
    }
    if (dhi[i] && at < p.capacity) p.ovr[at] = fdy_ovr32{byte_off + 4, (u32)(va[i] >> 32)};
    for (int w = 0; w < kDerBlock / 64; ++w) before += s_cnt[i][w];
  }
}

__global__ __launch_bounds__(1024) void derive_scan_kernel(DerParams p) {
  __shared__ u64 s_buf[17];
  const u32 n = *p.ws.n_tiles;
  u64 carry = 0;
  for (u32 j0 = 0; j0 < n; j0 += 1024) {
    const u32 j = j0 + threadIdx.x;
    const u64 c = j < n ? p.ws.tile_cnt[j] : 0;
    u64 total;
    const u64 e = block_excl_scan(c, s_buf, total);
    if (j < n) p.ws.tile_pos[j] = carry + e;
    carry += total;
  }
  __syncthreads();  // this workgroup's own tile_pos stores are read back below
  // a graph's offset: entries before its first tile (graphs without tiles included)
  for (u32 g = threadIdx.x; g <= p.n_graphs; g += 1024) {
    const u64 t = p.ws.tile_off[g];
    p.ovr_off[g] = t < n ? p.ws.tile_pos[t] : carry;
  }
  if (threadIdx.x == 0 && carry > p.capacity) raise_status(p.d_status, FDY_ST_CAPACITY);
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t layout(u64 n_words_total, u32 n_graphs, unsigned char* base, DerWs* ws) {
  const u64 max_tiles = n_words_total / kDerTile + n_graphs;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    unsigned char* p = base ? base + off : nullptr;
    off += align256(bytes);
    return p;
  };
  DerWs w;
  w.n_tiles = (u32*)take(4);
  w.tile_off = (u64*)take(((size_t)n_graphs + 1) * 8);
  w.tile_cnt = (u32*)take((size_t)max_tiles * 4);
  w.tile_pos = (u64*)take((size_t)max_tiles * 8);
  w.max_tiles = (u32)max_tiles;
  if (ws) *ws = w;
  return off;
}

bool sizes_ok(u64 n_words_total, u32 n_graphs) {
  return n_graphs <= (1u << 20) && n_words_total < (1ull << 40);
}

}  // namespace
}  // namespace fdy

using namespace fdy;

extern "C" size_t fdy_derive_workspace_bytes(uint64_t n_words_total, uint32_t n_graphs) {
  if (!sizes_ok(n_words_total, n_graphs)) return 0;
  return layout(n_words_total, n_graphs, nullptr, nullptr);
}

extern "C" int fdy_derive_overrides(const uint64_t* d_words, uint64_t n_words_total, const uint64_t* d_word_off,
                                    uint32_t n_graphs, const uint32_t* d_graph_tmpl,
                                    const uint32_t* d_tmpl_graph, uint32_t n_templates, fdy_ovr32* d_ovr,
                                    uint64_t ovr_capacity, uint64_t* d_ovr_off, void* d_workspace,
                                    size_t workspace_bytes, uint32_t* d_status, void* hip_stream) {
  if (!sizes_ok(n_words_total, n_graphs)) return FDY_ERR_INVALID_ARG;
  if (!d_word_off || !d_ovr_off) return FDY_ERR_INVALID_ARG;
  if (n_graphs && (!d_graph_tmpl || !d_tmpl_graph)) return FDY_ERR_INVALID_ARG;
  if (n_words_total && (!d_words || ((uintptr_t)d_words & 7))) return FDY_ERR_INVALID_ARG;
  if (ovr_capacity && (!d_ovr || ((uintptr_t)d_ovr & 7))) return FDY_ERR_INVALID_ARG;
  const size_t need = layout(n_words_total, n_graphs, nullptr, nullptr);
  if (!d_workspace || ((uintptr_t)d_workspace & 255) || workspace_bytes < need) return FDY_ERR_WORKSPACE;
  DerParams p;
  p.words = (const u64*)d_words;
  p.word_off = (const u64*)d_word_off;
  p.n_graphs = n_graphs;
  p.graph_tmpl = d_graph_tmpl;
  p.tmpl_graph = d_tmpl_graph;
  p.n_templates = n_templates;
  p.n_words_total = n_words_total;
  p.ovr = d_ovr;
  p.capacity = ovr_capacity;
  p.ovr_off = (u64*)d_ovr_off;
  p.d_status = d_status;
  layout(n_words_total, n_graphs, (unsigned char*)d_workspace, &p.ws);
  hipStream_t stream = (hipStream_t)hip_stream;
  (void)hipGetLastError();  // drop any stale error left by earlier, unrelated runtime calls
  hipLaunchKernelGGL(derive_prep_kernel, dim3(1), dim3(1024), 0, stream, p);
  FDY_HIP_TRY(hipGetLastError());
  if (p.ws.max_tiles) {
    hipLaunchKernelGGL(derive_tile_kernel<false>, dim3(p.ws.max_tiles), dim3(kDerBlock), 0, stream, p);
    FDY_HIP_TRY(hipGetLastError());
  }
  hipLaunchKernelGGL(derive_scan_kernel, dim3(1), dim3(1024), 0, stream, p);
  FDY_HIP_TRY(hipGetLastError());
  if (p.ws.max_tiles) {
    hipLaunchKernelGGL(derive_tile_kernel<true>, dim3(p.ws.max_tiles), dim3(kDerBlock), 0, stream, p);
    FDY_HIP_TRY(hipGetLastError());
  }
  return FDY_OK;
}
