// fdy_materialize.hip - (c) template materialization for gfx950.
//
// Section 4.2.1 prepares, at LOAD time, the parameter set of every non-template graph on
// CPU worker threads; Section 4.2.2 patches rank-dependent communication arguments.  Here
// the same preparation is one streaming pass on the GPU over all (base map, graph, tile)
// units, bounded by the HBM write of the output:
//
//   prep A (one workgroup)   prefix sums over the output graphs: where each graph's words,
//                            nodes and tiles start; verifies the caller's totals.  A launch
//                            of its own only above 1024 output graphs: up to there every
//                            block of prep B computes the sums itself, in LDS.
//   prep B (one launch)      three kinds of blocks side by side.  Tile blocks (one thread per
//                            tile) resolve each output tile once, independent of the base map:
//                            its graph, template, source words, and the sub-ranges of the
//                            template's relocation list and the graph's override list that
//                            fall inside the tile (a thread searches where its tile's ranges
//                            begin; they end where the next tile's begin).  Patch blocks (one
//                            thread per tile and rank) do the same for each rank's patch list.
//                            Dims blocks (one thread per node) write the launch dimensions of
//                            the template with the graph's grid overrides.  Plain per-lane
//                            binary searches: tens of thousands of them run side by side, and
//                            one request per halving is what the memory system serves best;
//                            the kernel's time is its longest chain of dependent loads.  One
//                            launch rather than four because small archives are bound by
//                            launch latency.
//   main  (tile x map group) stages the template tile in LDS and the tile's relocation entries
//                            in registers once, then per base map of its group scatters c2
//                            rebased pointers (new_base[m][region] + offset), c3 32-bit
//                            overrides and c4 64-bit rank patches into LDS in that order and
//                            streams the tile out with coalesced stores.  Templates,
//                            relocation lists and base maps are re-read per group from L2 /
//                            Infinity Cache; only the output is compulsory HBM traffic.
//   small launches           (every workgroup of main resident at once): no prep launch at
//                            all; each workgroup of main resolves its own tile first, and
//                            extra blocks of the same launch write the dimensions and check
//                            the short lists.  Same results, one launch less.
// The order of every list is verified on the way (FDY_ST_BAD_ORDER): the relocation lists
// where main reads them, the short lists by blocks of the prep launch (or of main).
#include <mutex>

#include "fdy_device.hpp"
#include "fdy_internal.h"

namespace fdy {
namespace {

constexpr int kMatTile = 2048;  // words per tile (16 KiB)
constexpr int kMatBlock = 256;

struct __attribute__((aligned(16))) MatTile {  // 64 B
  u64 src_word;  // index into src_words of the tile's first word
  u64 out_word;  // word offset of the tile inside one map's output
  u32 n_words;   // 0: unused entry
  u32 g, tmpl, k0;
  u32 reloc_lo, reloc_hi, ovr_lo, ovr_hi;
  u32 reloc_seg;  // first entry of the template's relocation list (order checks stop there)
  u32 pad[3];
};
static_assert(sizeof(MatTile) == 64, "MatTile");

struct MatHeader {
  u32 n_tiles;
  u32 ok;
};

struct MatWs {
  MatHeader* hdr;
  u64* out_word_off;  // [G+1]
  u64* out_node_off;  // [G+1]
  u64* tile_off;      // [G+1]
  MatTile* tiles;     // [max_tiles]
  uint2* tile_patch;  // [max_tiles * R]
  u32 max_tiles;
};

struct MatParams {
  fdy_mat_desc d;
  MatWs ws;
  u64* out_words;
  u32* out_dims;
  u32* d_status;
  u32 map_group;  // consecutive base maps handled by one workgroup of the main kernel
  u32 stream_once;  // templates and relocation lists are read once and too large to stay cached
};

// Word and node counts of output graph g (those of its template).  False, with zero counts, if
// its template or the template's source graph is out of range or has 2^32 words or more.
__device__ __forceinline__ bool graph_sizes(const MatParams& p, u32 g, u64& nw, u64& nn, u32* src_graph = nullptr) {
  const fdy_mat_desc& d = p.d;
  nw = 0;
  nn = 0;
  const u32 t = d.graph_tmpl[g];
  const u32 s = t < d.n_templates ? d.tmpl_graph[t] : 0xffffffffu;
  if (src_graph) *src_graph = s;
  if (s >= d.n_src_graphs) return false;
  nw = d.src_word_off[s + 1] - d.src_word_off[s];
  if (p.out_dims) nn = d.src_node_off[s + 1] - d.src_node_off[s];
  if (nw >> 32) {  // a template must stay below 2^32 words
    nw = 0;
    nn = 0;
    return false;
  }
  // a graph without words has no tile that would meet (and reject) its entries
  if (nw == 0 && (d.src_reloc_off[s + 1] != d.src_reloc_off[s] || d.ovr_off[g + 1] != d.ovr_off[g])) return false;
  return true;
}

// Do the totals match what the caller sized the launch and the outputs for?
__device__ __forceinline__ bool totals_ok(const MatParams& p, u64 words, u64 nodes, u64 tiles) {
  bool ok = words == p.d.out_words_per_map && tiles <= p.ws.max_tiles;
  if (p.out_dims && nodes != p.d.out_nodes_total) ok = false;
  return ok;
}

__global__ __launch_bounds__(1024) void mat_prep_graphs_kernel(MatParams p) {
  __shared__ u64 s_buf[17];
  const fdy_mat_desc& d = p.d;
  const u32 G = d.n_graphs;
  u64 carry_w = 0, carry_n = 0, carry_t = 0;
  bool bad = false;
  for (u32 g0 = 0; g0 < G; g0 += 1024) {
    const u32 g = g0 + threadIdx.x;
    u64 nw = 0, nn = 0;
    if (g < G && !graph_sizes(p, g, nw, nn)) bad = true;
    const u64 nt = (nw + kMatTile - 1) / kMatTile;
    u64 tw, tn, tt;
    const u64 ew = block_excl_scan(nw, s_buf, tw);
    const u64 en = block_excl_scan(nn, s_buf, tn);
    const u64 et = block_excl_scan(nt, s_buf, tt);
    if (g < G) {
      p.ws.out_word_off[g] = carry_w + ew;
      p.ws.out_node_off[g] = carry_n + en;
      p.ws.tile_off[g] = carry_t + et;
    }
    carry_w += tw;
    carry_n += tn;
    carry_t += tt;
  }
  if (bad) raise_status(p.d_status, FDY_ST_BAD_INDEX);
  if (threadIdx.x == 0) {
    p.ws.out_word_off[G] = carry_w;
    p.ws.out_node_off[G] = carry_n;
    p.ws.tile_off[G] = carry_t;
    const bool ok = totals_ok(p, carry_w, carry_n, carry_t);
    if (!ok) raise_status(p.d_status, FDY_ST_BAD_SIZE);
    p.ws.hdr->n_tiles = ok ? (u32)carry_t : 0u;
    p.ws.hdr->ok = ok ? 1u : 0u;
  }
}

// Per-lane lower bound: first index in [lo, hi) whose key is not below target (hi if none).
// One dependent load per halving; used where thousands of independent searches run side by
// side (one per lane), so that the memory system sees few requests per search.
template <typename KeyFn>
__device__ __forceinline__ u32 lane_lower_bound(KeyFn key, u32 lo, u32 hi, u64 target) {
  while (lo < hi) {
    const u32 mid = lo + ((hi - lo) >> 1);
    if (key(mid) < target) lo = mid + 1;
    else hi = mid;
  }
  return lo;
}

// Two per-lane lower bounds at once (A and B: independent lists), four-way: each step loads
// three keys per list, all six before any is used, so a list of n entries takes log4 n
// dependent round trips and the shorter search hides behind the longer one.  This kernel's
// time is its longest chain of dependent loads.
template <typename KeyA, typename KeyB>
__device__ __forceinline__ void lane_lower_bound_pair(KeyA key_a, u32 lo_a, u32 hi_a, u64 target_a, KeyB key_b,
                                                      u32 lo_b, u32 hi_b, u64 target_b, u32& res_a, u32& res_b) {
  while (lo_a < hi_a || lo_b < hi_b) {
    const u32 na = hi_a - lo_a, nb = hi_b - lo_b;
    // probe positions (ascending; equal ones for ranges below four entries are harmless)
    const u32 a1 = lo_a + na / 4, a2 = lo_a + na / 2, a3 = lo_a + na / 2 + na / 4;
    const u32 b1 = lo_b + nb / 4, b2 = lo_b + nb / 2, b3 = lo_b + nb / 2 + nb / 4;
    u64 ka1 = 0, ka2 = 0, ka3 = 0, kb1 = 0, kb2 = 0, kb3 = 0;
    if (na) {
      ka1 = key_a(a1);
      ka2 = key_a(a2);
      ka3 = key_a(a3);
    }
    if (nb) {
      kb1 = key_b(b1);
      kb2 = key_b(b2);
      kb3 = key_b(b3);
    }
    if (na) {
      if (ka3 < target_a) lo_a = a3 + 1;
      else if (ka2 < target_a) { lo_a = a2 + 1; hi_a = a3; }
      else if (ka1 < target_a) { lo_a = a1 + 1; hi_a = a2; }
      else hi_a = a1;
    }
    if (nb) {
      if (kb3 < target_b) lo_b = b3 + 1;
      else if (kb2 < target_b) { lo_b = b2 + 1; hi_b = b3; }
      else if (kb1 < target_b) { lo_b = b1 + 1; hi_b = b2; }
      else hi_b = b1;
    }
  }
  res_a = lo_a;
  res_b = lo_b;
}

// The per-graph prefix sums as the tile, patch and dims blocks read them: from the workspace
// (written by mat_prep_graphs_kernel) or from the block's own LDS copy.
struct PrepView {
  const u64* out_word_off;  // [G+1]
  const u64* out_node_off;  // [G+1]
  const u64* tile_off;      // [G+1]
  u32 n_tiles;              // 0 if the totals do not match
  u32 ok;
};

// Where tile j (j < n_tiles) lies: its graph, template, source graph, first word inside the
// graph, word count, first source word, and whether it is the graph's last tile.
struct TileGeom {
  u32 g, t, s, n;
  u64 k0, src_word;
  bool last;
};
__device__ __forceinline__ TileGeom tile_geometry(const MatParams& p, const PrepView& v, u32 j) {
  const fdy_mat_desc& d = p.d;
  const u64* tile_off = v.tile_off;
  TileGeom q;
  // largest g with tile_off[g] <= j
  q.g = lane_lower_bound([&](u32 i) { return tile_off[i]; }, 0u, d.n_graphs + 1u, (u64)j + 1) - 1;
  q.t = d.graph_tmpl[q.g];
  q.s = d.tmpl_graph[q.t];  // valid: graphs with a bad template have no tiles
  const u64 w0 = d.src_word_off[q.s];
  const u64 nw = d.src_word_off[q.s + 1] - w0;
  q.k0 = ((u64)j - tile_off[q.g]) * kMatTile;
  q.n = (u32)((nw - q.k0) < (u64)kMatTile ? (nw - q.k0) : (u64)kMatTile);
  q.src_word = w0 + q.k0;
  q.last = q.k0 + q.n == nw;
  return q;
}

// A block of 256 threads resolves kPrepTiles = 255 consecutive output tiles (independent of the
// base map).  Every thread finds where its tile's slices of the template's relocation list
// and of the graph's override list BEGIN; where they end is where the next tile's begin (the
// next thread's result, through LDS) or, for a graph's last tile, the end of the list.  That
// halves the chain of dependent loads, which is all this kernel's time.  Thread 255 only
// supplies the begins of the tile after the block's last.  Both ends stay bounded by the tile
// size, so a malformed list can never index outside what mat_main_kernel reserves; entries
// that do not belong to the tile are caught there.
constexpr u32 kPrepTiles = 255;
__device__ __forceinline__ void prep_tiles_block(const MatParams& p, const PrepView& v, u32 block, uint2* s_lo) {
  const fdy_mat_desc& d = p.d;
  const u32 tid = threadIdx.x;
  const u32 j = block * kPrepTiles + tid;
  const bool valid = j < v.n_tiles;
  TileGeom q;
  u32 rl0 = 0, rl1 = 0, ov1 = 0, reloc_lo = 0, ovr_lo = 0;
  if (valid) {
    q = tile_geometry(p, v, j);
    const fdy_reloc* relocs = d.relocs;
    rl0 = (u32)d.src_reloc_off[q.s];
    rl1 = (u32)d.src_reloc_off[q.s + 1];
    const fdy_ovr32* ovr = d.ovr;
    const u32 ov0 = (u32)d.ovr_off[q.g];
    ov1 = (u32)d.ovr_off[q.g + 1];
    lane_lower_bound_pair([&](u32 i) { return (u64)relocs[i].word; }, rl0, rl1, q.src_word,
                          [&](u32 i) { return (u64)ovr[i].byte_off; }, ov0, ov1, q.k0 * 8, reloc_lo, ovr_lo);
  }
  s_lo[tid] = make_uint2(reloc_lo, ovr_lo);
  __syncthreads();
  if (tid >= kPrepTiles || j >= p.ws.max_tiles) return;
  MatTile* ent = &p.ws.tiles[j];
  if (!valid) {
    ent->n_words = 0;
    return;
  }
  // a tile that is not its graph's last is followed by a tile of the same graph (j + 1 < n_tiles)
  u32 reloc_hi = q.last ? rl1 : s_lo[tid + 1].x;
  const u32 ovr_hi = q.last ? ov1 : s_lo[tid + 1].y;
  // the list is strictly ascending by word: at most n entries fall inside the tile, and none
  // lies before the template's first word
  if (reloc_hi - reloc_lo > q.n) {
    reloc_hi = reloc_lo + q.n;
    raise_status(p.d_status, FDY_ST_BAD_ORDER);
  }
  if (q.k0 == 0 && reloc_lo != rl0) raise_status(p.d_status, FDY_ST_BAD_INDEX);
  MatTile e;
  e.src_word = q.src_word;
  e.out_word = v.out_word_off[q.g] + q.k0;
  e.n_words = q.n;
  e.g = q.g;
  e.tmpl = q.t;
  e.k0 = (u32)q.k0;
  e.reloc_lo = reloc_lo;
  e.reloc_hi = reloc_hi;
  e.ovr_lo = ovr_lo;
  e.ovr_hi = ovr_hi;
  e.reloc_seg = rl0;
  e.pad[0] = e.pad[1] = e.pad[2] = 0;
  *ent = e;
}

// Thread i: (output tile, rank) pair i: the slice of the rank's patch list inside the tile.
// Works from the tile's geometry, not from the tile table, which the same launch is writing.
__device__ __forceinline__ void prep_patch(const MatParams& p, const PrepView& v, u64 i) {
  const fdy_mat_desc& d = p.d;
  const u32 R = d.n_ranks;
  if (i >= (u64)v.n_tiles * R) return;
  const u32 j = (u32)(i / R), r = (u32)(i % R);
  const TileGeom e = tile_geometry(p, v, j);
  const fdy_patch* patch = d.patch;
  const u64 row = (u64)e.t * R + r;
  const u32 p0 = (u32)d.patch_off[row], p1 = (u32)d.patch_off[row + 1];
  const u32 lo = lane_lower_bound([&](u32 q) { return (u64)patch[q].word; }, p0, p1, e.k0);
  const u32 hi = lane_lower_bound([&](u32 q) { return (u64)patch[q].word; }, lo, p1, e.k0 + e.n);
  p.ws.tile_patch[i] = make_uint2(lo, hi);
}

// Stage the template tile in LDS: 16-byte global loads from the first even word on.
__device__ __forceinline__ void stage_tile(u64* buf, const u64* src, u64 src_word, u32 n, u32 tid, bool once) {
  typedef u64 v2u64 __attribute__((ext_vector_type(2)));
  const u32 head = (u32)(src_word & 1);  // words before 16-byte alignment (n >= 1 here)
  const u32 pairs = (n - head) >> 1;
  if (tid == 0 && head) buf[0] = src[0];
  if (once) {
    for (u32 i = tid; i < pairs; i += kMatBlock) {
      const v2u64 v = __builtin_nontemporal_load(reinterpret_cast<const v2u64*>(src + head + 2 * i));
      buf[head + 2 * i] = v.x;
      buf[head + 2 * i + 1] = v.y;
    }
  } else {
    for (u32 i = tid; i < pairs; i += kMatBlock) {
      const u64x2 v = *reinterpret_cast<const u64x2*>(src + head + 2 * i);
      buf[head + 2 * i] = v.x;
      buf[head + 2 * i + 1] = v.y;
    }
  }
  if (tid == 0 && head + 2 * pairs < n) buf[n - 1] = src[n - 1];
}

// The same in two steps, so that other work can sit between the loads and their use (the
// self-resolving form of the main kernel searches its slices meanwhile).
constexpr int kTileChunks = kMatTile / (2 * kMatBlock);
struct TileRegs {
  u64x2 v[kTileChunks];
  u64 first, last;
};
__device__ __forceinline__ void tile_load(TileRegs& r, const u64* src, u64 src_word, u32 n, u32 tid, bool once) {
  typedef u64 v2u64 __attribute__((ext_vector_type(2)));
  const u32 head = (u32)(src_word & 1);  // words before 16-byte alignment (n >= 1 here)
  const u32 pairs = (n - head) >> 1;
  r.first = r.last = 0;
  if (tid == 0 && head) r.first = src[0];
#pragma unroll
  for (int c = 0; c < kTileChunks; ++c) {
    const u32 i = tid + (u32)c * kMatBlock;
    r.v[c] = u64x2{0, 0};
    if (i < pairs) {
      if (once) {
        const v2u64 v = __builtin_nontemporal_load(reinterpret_cast<const v2u64*>(src + head + 2 * i));
        r.v[c].x = v.x;
        r.v[c].y = v.y;
      } else {
        r.v[c] = *reinterpret_cast<const u64x2*>(src + head + 2 * i);
      }
    }
  }
  if (tid == 0 && head + 2 * pairs < n) r.last = src[n - 1];
}
__device__ __forceinline__ void tile_store(u64* buf, const TileRegs& r, u64 src_word, u32 n, u32 tid) {
  const u32 head = (u32)(src_word & 1);
  const u32 pairs = (n - head) >> 1;
  if (tid == 0 && head) buf[0] = r.first;
#pragma unroll
  for (int c = 0; c < kTileChunks; ++c) {
    const u32 i = tid + (u32)c * kMatBlock;
    if (i < pairs) {
      buf[head + 2 * i] = r.v[c].x;
      buf[head + 2 * i + 1] = r.v[c].y;
    }
  }
  if (tid == 0 && head + 2 * pairs < n) buf[n - 1] = r.last;
}

// Order of the short lists (overrides, grid overrides, rank patches): every entry against the
// one before it, all lists of a kind in one sweep over their concatenation; where the key does
// not ascend, a new list must begin.  The relocation lists, which are long, are checked where
// they are read anyway (mat_main_kernel).
__device__ __forceinline__ void check_lists(const MatParams& p, u32 cb, u32 n_cb) {
  const fdy_mat_desc& d = p.d;
  const u64 first = (u64)cb * 256 + threadIdx.x, stride = (u64)n_cb * 256;
  bool disorder = false;
  auto sweep = [&](auto key, const u64* off, u32 n_lists) {
    if (!n_lists) return;
    const u64 lo = off[0], hi = off[n_lists];
    for (u64 i = lo + 1 + first; i < hi; i += stride) {
      if (key(i - 1) < key(i)) continue;
      u32 a = 0, b = n_lists;  // the last list that begins at or before entry i
      while (b - a > 1) {
        const u32 mid = a + (b - a) / 2;
        if (off[mid] <= i) a = mid;
        else b = mid;
      }
      if (off[a] != i) disorder = true;
    }
  };
  const fdy_ovr32* ovr = d.ovr;
  sweep([&](u64 i) { return ovr[i].byte_off; }, d.ovr_off, d.n_graphs);
  if (p.out_dims) {
    const fdy_grid_ovr* govr = d.govr;
    sweep([&](u64 i) { return govr[i].node; }, d.govr_off, d.n_graphs);
  }
  if (d.map_rank) {
    const fdy_patch* patch = d.patch;
    sweep([&](u64 i) { return patch[i].word; }, d.patch_off, d.n_templates * d.n_ranks);
  }
  if (disorder) raise_status(p.d_status, FDY_ST_BAD_ORDER);
}

// Thread i: launch dimensions of output node i.
__device__ __forceinline__ void write_dims(const MatParams& p, const PrepView& v, u64 i) {
  const fdy_mat_desc& d = p.d;
  if (!v.ok) return;
  if (i >= d.out_nodes_total) return;
  // largest g with out_node_off[g] <= i
  const u64* off = v.out_node_off;
  u32 lo = 0, hi = d.n_graphs;  // answer in [lo, hi)
  while (hi - lo > 1) {
    const u32 mid = lo + (hi - lo) / 2;
    if (off[mid] <= i) lo = mid;
    else hi = mid;
  }
  const u32 g = lo;
  const u32 n = (u32)(i - off[g]);
  const u32 s = d.tmpl_graph[d.graph_tmpl[g]];
  const fdy_node nd = d.src_nodes[d.src_node_off[s] + n];
  u32 gx = nd.grid[0], gy = nd.grid[1], gz = nd.grid[2];
  // grid override of this node, if any (list ascending by node)
  u64 a = d.govr_off[g], b = d.govr_off[g + 1];
  while (a < b) {
    const u64 mid = a + (b - a) / 2;
    if (d.govr[mid].node < n) a = mid + 1;
    else b = mid;
  }
  if (a < d.govr_off[g + 1] && d.govr[a].node == n) {
    gx = d.govr[a].grid[0];
    gy = d.govr[a].grid[1];
    gz = d.govr[a].grid[2];
  }
  uint2* o = reinterpret_cast<uint2*>(p.out_dims + i * 6);
  o[0] = make_uint2(gx, gy);
  o[1] = make_uint2(gz, nd.block[0]);
  o[2] = make_uint2(nd.block[1], nd.block[2]);
}

// One workgroup per (tile, group of consecutive base maps).  What does not depend on the map
// is fetched once per workgroup: the tile entry, the template tile (LDS) and this thread's
// share of the tile's relocation entries (registers; the slice holds at most kMatTile
// entries, kMatPre per thread).  Per map only the base-map gathers, the scatter into LDS
// and the store of the tile repeat.  Relocations and overrides hit the same words for every
// map, so the LDS copy needs no refresh between maps; rank patches differ per map, so the
// words the previous map's rank patched are given their template values back first.
constexpr int kMatPre = kMatTile / kMatBlock;
constexpr int kMatStore = kMatTile / (2 * kMatBlock);  // 16-byte chunks per thread
constexpr int kMatOvrPre = 2;                          // overrides of the tile a thread keeps in registers

//
// kSelf (small launches: every workgroup resident at once, at most kSelfGraphs output graphs):
// no tile table exists; the workgroup works out its own tile first (per-graph prefix sums in
// LDS, then its slices of the lists, one cooperative search per wave), and further blocks of
// the same launch write the launch dimensions and check the order of the short lists.  That
// is mat_prep_tiles_kernel's work without its launch: the model-shaped archives are bound by
// launches, and an extra 4 us of prologue in workgroups that all run side by side is less than
// the 10 us the launch costs.
constexpr u32 kSelfGraphs = 1000;   // offsets of up to 1,024 graphs fit the tile buffer
constexpr u32 kSelfMaxGroup = 8;    // most base maps per workgroup in this mode

// Per-graph sums of a kSelf block, in the 16 KiB tile buffer: tile_off u32[1024] | source graph
// u32[1024] | out_word_off (or, for the blocks that write dimensions, out_node_off) u64[1024].
// Returns whether the totals match what the caller sized the launch for; `bad` reports an
// output graph without a valid template.
struct SelfSums {
  u32* tile_off;
  u32* src;
  u64* off;
  u32 n_tiles;
  bool ok, bad;
};
__device__ __forceinline__ SelfSums self_sums(const MatParams& p, u64* buf, u64* s_buf, bool nodes) {
  SelfSums r;
  r.tile_off = reinterpret_cast<u32*>(buf);
  r.src = r.tile_off + 1024;
  r.off = buf + 1024;
  const u32 G = p.d.n_graphs, tid = threadIdx.x;
  constexpr u32 kPer = 1024 / kMatBlock;
  u64 nw[kPer], nn[kPer], sum_w = 0, sum_n = 0, sum_t = 0;
  u32 from[kPer];
  bool bad = false;
#pragma unroll
  for (u32 i = 0; i < kPer; ++i) {
    const u32 g = tid * kPer + i;
    nw[i] = 0;
    nn[i] = 0;
    from[i] = 0;
    if (g < G && !graph_sizes(p, g, nw[i], nn[i], &from[i])) bad = true;
    sum_w += nw[i];
    sum_n += nn[i];
    sum_t += (nw[i] + kMatTile - 1) / kMatTile;
  }
  u64 tw, tn, tt;
  u64 ew = block_excl_scan(sum_w, s_buf, tw);
  u64 en = block_excl_scan(sum_n, s_buf, tn);
  u64 et = block_excl_scan(sum_t, s_buf, tt);
#pragma unroll
  for (u32 i = 0; i < kPer; ++i) {
    const u32 g = tid * kPer + i;
    if (g < G) {
      r.tile_off[g] = (u32)et;
      r.src[g] = from[i];
      r.off[g] = nodes ? en : ew;
    }
    ew += nw[i];
    en += nn[i];
    et += (nw[i] + kMatTile - 1) / kMatTile;
  }
  if (tid == 0) {
    r.tile_off[G] = (u32)tt;
    r.off[G] = nodes ? tn : tw;
  }
  r.ok = totals_ok(p, tw, tn, tt);
  r.n_tiles = r.ok ? (u32)tt : 0u;
  r.bad = __syncthreads_or(bad);
  return r;
}

template <bool kSelf>
__global__ __launch_bounds__(kMatBlock) void mat_main_kernel(MatParams p, u32 n_tile_blocks, u32 nb_dims) {
  __shared__ __align__(16) u64 buf[kMatTile];
  __shared__ u64 s_buf[kSelf ? 17 : 1];
  __shared__ u32 s_found[kSelf ? 4 + 2 * kSelfMaxGroup : 1];
  typedef u64 v2u64 __attribute__((ext_vector_type(2)));
  const fdy_mat_desc& d = p.d;
  const u32 j = blockIdx.x, tid = threadIdx.x;
  const u32 m0 = blockIdx.y * p.map_group;
  const u32 m1 = min(m0 + p.map_group, d.n_maps);
  // Template words and relocation entries that no other map group reads again, in an archive
  // too large to stay in the L2s anyway (the host decides: one map group, and from 4,096 tiles
  // = 64 MiB on, twice the chip's L2s), are loaded non-temporally, so that the base map keeps
  // its place in L2 for the gathers (config 4: 0.51 -> 0.47 ms); small archives stay cached for
  // whoever reads them next.
  const bool once = p.stream_once != 0;
  MatTile ent;
  if constexpr (kSelf) {
    if (j >= n_tile_blocks) {  // launch dimensions, then the order of the short lists
      if (blockIdx.y) return;
      if (j < n_tile_blocks + nb_dims) {
        const SelfSums q = self_sums(p, buf, s_buf, true);
        PrepView v;
        v.out_word_off = nullptr;
        v.out_node_off = q.off;
        v.tile_off = nullptr;
        v.n_tiles = q.n_tiles;
        v.ok = q.ok ? 1u : 0u;
        write_dims(p, v, (u64)(j - n_tile_blocks) * kMatBlock + tid);
      } else {
        check_lists(p, j - n_tile_blocks - nb_dims, gridDim.x - n_tile_blocks - nb_dims);
      }
      return;
    }
    const SelfSums q = self_sums(p, buf, s_buf, false);
    if (j == 0 && blockIdx.y == 0) {  // what the prep launch reports
      if (q.bad) raise_status(p.d_status, FDY_ST_BAD_INDEX);
      if (tid == 0 && !q.ok) raise_status(p.d_status, FDY_ST_BAD_SIZE);
    }
    if (j >= q.n_tiles) return;
    // the tile's graph: the last one whose first tile is not behind tile j
    u32 glo = 0, ghi = d.n_graphs;  // answer in [glo, ghi)
    while (ghi - glo > 1) {
      const u32 mid = glo + (ghi - glo) / 2;
      if (q.tile_off[mid] <= j) glo = mid;
      else ghi = mid;
    }
    const u32 g = glo, s_graph = q.src[g];
    const u32 k0 = (j - q.tile_off[g]) * (u32)kMatTile;
    const u64 out_word = q.off[g] + k0;
    const u32 nw = (u32)(q.off[g + 1] - q.off[g]);  // a template stays below 2^32 words
    const u32 n_here = min(nw - k0, (u32)kMatTile);
    const bool last = k0 + n_here == nw;
    const u32 t = d.graph_tmpl[g];
    const u64 src_word = d.src_word_off[s_graph] + k0;
    const u32 rl0 = (u32)d.src_reloc_off[s_graph], rl1 = (u32)d.src_reloc_off[s_graph + 1];
    const u32 ov0 = (u32)d.ovr_off[g], ov1 = (u32)d.ovr_off[g + 1];
    __syncthreads();  // everyone has read the sums; the buffer is free for the tile
    TileRegs tile;
    tile_load(tile, d.src_words + src_word, src_word, n_here, tid, once);  // in flight during the searches
    {
      // one cooperative search per wave: where the tile's slices of the template's relocation
      // list and of the graph's override list begin and end; then the patch slices of the
      // group's maps, two searches each
      const u32 w = tid >> 6;
      const fdy_reloc* relocs = d.relocs;
      const fdy_ovr32* ovr = d.ovr;
      u32 r = 0;
      if (w == 0) r = wave_lower_bound([&](u32 i) { return (u64)relocs[i].word; }, rl0, rl1, src_word);
      if (w == 1) r = last ? rl1 : wave_lower_bound([&](u32 i) { return (u64)relocs[i].word; }, rl0, rl1, src_word + n_here);
      if (w == 2) r = wave_lower_bound([&](u32 i) { return (u64)ovr[i].byte_off; }, ov0, ov1, (u64)k0 * 8);
      if (w == 3) r = last ? ov1 : wave_lower_bound([&](u32 i) { return (u64)ovr[i].byte_off; }, ov0, ov1, ((u64)k0 + n_here) * 8);
      if (lane_id() == 0) s_found[w] = r;
      if (d.map_rank) {
        const fdy_patch* patch = d.patch;
        for (u32 e = w; e < 2 * (m1 - m0); e += kMatBlock / 64) {
          const u32 rank = d.map_rank[m0 + (e >> 1)];
          u32 f = (e & 1) ? 0u : 0xffffffffu;  // a bad rank: the slice that mat_main takes for "none, and flag it"
          if (rank < d.n_ranks) {
            const u64 row = (u64)t * d.n_ranks + rank;
            const u32 p0 = (u32)d.patch_off[row], p1 = (u32)d.patch_off[row + 1];
            f = wave_lower_bound([&](u32 i) { return (u64)patch[i].word; }, p0, p1, (u64)k0 + ((e & 1) ? n_here : 0u));
          }
          if (lane_id() == 0) s_found[4 + e] = f;
        }
      }
    }
    tile_store(buf, tile, src_word, n_here, tid);  // c1
    __syncthreads();
    ent.src_word = src_word;
    ent.out_word = out_word;
    ent.n_words = n_here;
    ent.g = g;
    ent.tmpl = t;
    ent.k0 = k0;
    ent.reloc_lo = s_found[0];
    ent.reloc_hi = s_found[1];
    ent.ovr_lo = s_found[2];
    ent.ovr_hi = s_found[3];
    ent.reloc_seg = rl0;
    if (ent.reloc_hi < ent.reloc_lo) ent.reloc_hi = ent.reloc_lo;  // (a list out of order can cross them)
    if (ent.ovr_hi < ent.ovr_lo) ent.ovr_hi = ent.ovr_lo;
    if (ent.reloc_hi - ent.reloc_lo > n_here) {  // strictly ascending: at most one entry per word
      ent.reloc_hi = ent.reloc_lo + n_here;
      if (blockIdx.y == 0) raise_status(p.d_status, FDY_ST_BAD_ORDER);
    }
    if (k0 == 0 && ent.reloc_lo != rl0 && blockIdx.y == 0) raise_status(p.d_status, FDY_ST_BAD_INDEX);
  } else {
    ent = p.ws.tiles[j];
  }
  const u32 n = ent.n_words;
  if (n == 0) return;
  const u64* src = d.src_words + ent.src_word;
  if constexpr (!kSelf) stage_tile(buf, src, ent.src_word, n, tid, once);  // c1
  bool bad = false, disorder = false;
  u32 rk[kMatPre], rr[kMatPre];
  u64 ro[kMatPre];
#pragma unroll
  for (int i = 0; i < kMatPre; ++i) {
    const u32 q = ent.reloc_lo + tid + (u32)i * kMatBlock;
    rk[i] = 0xffffffffu;
    rr[i] = 0;
    ro[i] = 0;
    u32 word_q = 0;
    if (q < ent.reloc_hi) {
      u64x2 raw;
      if (once) {
        typedef u64 v2u64 __attribute__((ext_vector_type(2)));
        const v2u64 r = __builtin_nontemporal_load(reinterpret_cast<const v2u64*>(&d.relocs[q]));
        raw.x = r.x;
        raw.y = r.y;
      } else {
        raw = *reinterpret_cast<const u64x2*>(&d.relocs[q]);
      }
      const u32 word = (u32)raw.x, region = (u32)(raw.x >> 32);
      word_q = word;
      const u64 k = (u64)word - ent.src_word;
      if (k < n && region < d.n_alloc) {
        rk[i] = (u32)k;
        rr[i] = region;
        ro[i] = raw.y;
      } else {
        bad = true;
      }
    }
    // Strictly ascending by word: every entry of the slice against the one before it in the
    // template's list (the lower lane holds it; a wave's first lane reads it).  The slices of a
    // template's tiles cover its list, so a list that passes everywhere is in order, which is
    // what the slices themselves (found by binary search) rely on.
    u32 before = __shfl_up(word_q, 1);
    if (q < ent.reloc_hi && q > ent.reloc_seg) {
      if (lane_id() == 0) before = d.relocs[q - 1].word;
      if (before >= word_q) disorder = true;
    }
  }
  const bool has_ovr = ent.ovr_lo < ent.ovr_hi;
  const bool has_patch = d.map_rank != nullptr;
  // What repeats per map is kept off the chain of dependent loads as far as it goes: the
  // tile's overrides (the same for every map) wait in registers, kMatOvrPre per thread; a map's
  // patch slice is looked up one map ahead; its entries are requested together with the base-map
  // gathers, one per thread; and a patched word gets back what it held before the patch (the
  // template's value, or a rebased or overridden one that the next map's c2 / c3 write again
  // anyway) from a register instead of from the template in memory.  Lists longer than the
  // registers hold take their surplus from memory, in the same stage.
  u32 ov_at[kMatOvrPre], ov_val[kMatOvrPre];
  if (has_ovr) {
#pragma unroll
    for (int i = 0; i < kMatOvrPre; ++i) {
      const u32 q = ent.ovr_lo + tid + (u32)i * kMatBlock;
      ov_at[i] = 0xffffffffu;
      ov_val[i] = 0;
      if (q < ent.ovr_hi) {
        const fdy_ovr32 o = d.ovr[q];
        const u64 b = (u64)o.byte_off - (u64)ent.k0 * 8;
        if ((b >> 3) < n && (b & 3) == 0) {
          ov_at[i] = (u32)(b >> 2);
          ov_val[i] = o.value;
        } else {
          bad = true;
        }
      }
    }
  }
  auto patch_slice = [&](u32 m) {  // the slice of map m's rank inside this tile; empty for a bad rank
    if constexpr (kSelf) {
      const u32 lo = s_found[4 + 2 * (m - m0)], hi = s_found[5 + 2 * (m - m0)];
      return make_uint2(lo, lo == 0xffffffffu ? 0u : max(hi, lo));
    } else {
      const u32 rk_m = d.map_rank[m];
      return rk_m < d.n_ranks ? p.ws.tile_patch[(u64)j * d.n_ranks + rk_m] : make_uint2(0xffffffffu, 0);
    }
  };
  // this thread's patch entry of a slice (none: word index all ones)
  auto patch_entry = [&](uint2 pr) {
    u64x2 e = u64x2{~0ull, 0};
    if (pr.x != 0xffffffffu && pr.x + tid < pr.y) e = *reinterpret_cast<const u64x2*>(&d.patch[pr.x + tid]);
    return e;
  };
  uint2 pr_next = has_patch ? patch_slice(m0) : make_uint2(0, 0);
  u64x2 pe_next = has_patch ? patch_entry(pr_next) : u64x2{~0ull, 0};
  __syncthreads();
  for (u32 m = m0; m < m1; ++m) {
    const uint2 pr = pr_next;
    const u64x2 pe = pe_next;
    if (has_patch && m + 1 < m1) {
      pr_next = patch_slice(m + 1);
      pe_next = patch_entry(pr_next);
    }
    // requests of this map: the base-map gathers (c2); its patch entry (c4) came a map ahead
    const u64* nb = d.new_base + (u64)m * d.n_alloc;
    u64 base[kMatPre];
#pragma unroll
    for (int i = 0; i < kMatPre; ++i) base[i] = rk[i] != 0xffffffffu ? nb[rr[i]] : 0;
    const bool my_patch = has_patch && (u32)pe.x != 0xffffffffu;
    if (has_patch && pr.x == 0xffffffffu) bad = true;
    // c2: rebase
#pragma unroll
    for (int i = 0; i < kMatPre; ++i)
      if (rk[i] != 0xffffffffu) buf[rk[i]] = base[i] + ro[i];
    // c3: 32-bit overrides
    if (has_ovr) {
      __syncthreads();
      u32* buf32 = reinterpret_cast<u32*>(buf);
#pragma unroll
      for (int i = 0; i < kMatOvrPre; ++i)
        if (ov_at[i] != 0xffffffffu) buf32[ov_at[i]] = ov_val[i];
      for (u32 q = ent.ovr_lo + tid + kMatOvrPre * kMatBlock; q < ent.ovr_hi; q += kMatBlock) {
        const fdy_ovr32 o = d.ovr[q];
        const u64 b = (u64)o.byte_off - (u64)ent.k0 * 8;
        if ((b >> 3) < n && (b & 3) == 0) buf32[b >> 2] = o.value;
        else bad = true;
      }
    }
    // c4: rank patches; what the patched word held goes to a register for the way back
    u32 undo_at = 0xffffffffu;
    u64 undo_val = 0;
    const bool long_slice = has_patch && pr.x != 0xffffffffu && pr.y - pr.x > (u32)kMatBlock;
    if (has_patch) {
      __syncthreads();
      if (my_patch) {
        const u64 k = (u64)(u32)pe.x - ent.k0;
        if (k < n) {
          undo_at = (u32)k;
          undo_val = buf[k];
          buf[k] = pe.y;
        } else {
          bad = true;
        }
      }
      if (long_slice)
        for (u32 q = pr.x + tid + kMatBlock; q < pr.y; q += kMatBlock) {
          const u64x2 raw = *reinterpret_cast<const u64x2*>(&d.patch[q]);
          const u64 k = (u64)(u32)raw.x - ent.k0;
          if (k < n) buf[k] = raw.y;
          else bad = true;
        }
    }
    __syncthreads();
    // stream the tile out: LDS -> registers, then 16-byte non-temporal stores (the output is
    // written once and not read again here; keeping it out of L2 leaves the templates, lists
    // and base maps there).  The barrier sits between the LDS reads and the global stores so
    // that the next map's scatter can start while the stores drain.
    const u64 out_at = (u64)m * d.out_words_per_map + ent.out_word;
    u64* out = p.out_words + out_at;
    const u32 head = (u32)(out_at & 1);
    const u32 pairs = (n - head) >> 1;
    v2u64 v[kMatStore];
#pragma unroll
    for (int c = 0; c < kMatStore; ++c) {
      const u32 i = tid + (u32)c * kMatBlock;
      if (i < pairs) {
        v[c].x = buf[head + 2 * i];
        v[c].y = buf[head + 2 * i + 1];
      }
    }
    const u64 first = buf[0], last = buf[n - 1];
    if (m + 1 < m1) {
      __syncthreads();
      if (has_patch) {
        // the patched words get back what they held (the surplus of a long slice: the template's
        // value from memory); relocations and overrides that touch them are applied again
        if (undo_at != 0xffffffffu) buf[undo_at] = undo_val;
        if (long_slice)
          for (u32 q = pr.x + tid + kMatBlock; q < pr.y; q += kMatBlock) {
            const u64 k = (u64)d.patch[q].word - ent.k0;
            if (k < n) buf[k] = src[k];
          }
        __syncthreads();
      }
    }
#pragma unroll
    for (int c = 0; c < kMatStore; ++c) {
      const u32 i = tid + (u32)c * kMatBlock;
      if (i < pairs) __builtin_nontemporal_store(v[c], reinterpret_cast<v2u64*>(out + head + 2 * i));
    }
    if (tid == 0 && head) __builtin_nontemporal_store(first, out);
    if (tid == 0 && head + 2 * pairs < n) __builtin_nontemporal_store(last, out + n - 1);
  }
  if (bad) raise_status(p.d_status, FDY_ST_BAD_INDEX);
  if (disorder) raise_status(p.d_status, FDY_ST_BAD_ORDER);
}

// Everything that only needs the per-graph prefix sums, in one launch (these are small and
// launch-bound: three launches cost three times one): blocks [0, nb_tiles) resolve tiles,
// the next nb_patch blocks the (tile, rank) patch slices, the rest write launch dimensions.
// kOwnSums (at most kOwnSumsMax output graphs): every block computes the prefix sums itself,
// in LDS, instead of reading what mat_prep_graphs_kernel left in the workspace; that launch
// is then not needed at all.  Block 0 reports what that kernel would have reported.
constexpr u32 kOwnSumsMax = 1024;
constexpr u32 kCheckBlocks = 96;
template <bool kOwnSums>
__global__ __launch_bounds__(256) void mat_prep_tiles_kernel(MatParams p, u32 nb_tiles, u32 nb_patch) {
  if (blockIdx.x >= gridDim.x - kCheckBlocks) {  // the last blocks verify the order of the short lists
    check_lists(p, blockIdx.x - (gridDim.x - kCheckBlocks), kCheckBlocks);
    return;
  }
  __shared__ uint2 s_lo[256];
  __shared__ u64 s_off[kOwnSums ? 3 : 1][kOwnSums ? kOwnSumsMax + 1 : 1];
  __shared__ u64 s_buf[17];
  PrepView v;
  if constexpr (kOwnSums) {
    const u32 G = p.d.n_graphs, tid = threadIdx.x;
    constexpr u32 kPer = kOwnSumsMax / 256;
    u64 nw[kPer], nn[kPer], sum_w = 0, sum_n = 0, sum_t = 0;
    bool bad = false;
#pragma unroll
    for (u32 i = 0; i < kPer; ++i) {
      const u32 g = tid * kPer + i;
      nw[i] = 0;
      nn[i] = 0;
      if (g < G && !graph_sizes(p, g, nw[i], nn[i])) bad = true;
      sum_w += nw[i];
      sum_n += nn[i];
      sum_t += (nw[i] + kMatTile - 1) / kMatTile;
    }
    u64 tw, tn, tt;
    u64 ew = block_excl_scan(sum_w, s_buf, tw);
    u64 en = block_excl_scan(sum_n, s_buf, tn);
    u64 et = block_excl_scan(sum_t, s_buf, tt);
#pragma unroll
    for (u32 i = 0; i < kPer; ++i) {
      const u32 g = tid * kPer + i;
      if (g < G) {
        s_off[0][g] = ew;
        s_off[1][g] = en;
        s_off[2][g] = et;
      }
      ew += nw[i];
      en += nn[i];
      et += (nw[i] + kMatTile - 1) / kMatTile;
    }
    if (tid == 0) {
      s_off[0][G] = tw;
      s_off[1][G] = tn;
      s_off[2][G] = tt;
    }
    __syncthreads();
    const bool ok = totals_ok(p, tw, tn, tt);
    v.out_word_off = s_off[0];
    v.out_node_off = s_off[1];
    v.tile_off = s_off[2];
    v.n_tiles = ok ? (u32)tt : 0u;
    v.ok = ok ? 1u : 0u;
    if (blockIdx.x == 0) {
      if (bad) raise_status(p.d_status, FDY_ST_BAD_INDEX);
      if (tid == 0 && !ok) raise_status(p.d_status, FDY_ST_BAD_SIZE);
    }
  } else {
    v.out_word_off = p.ws.out_word_off;
    v.out_node_off = p.ws.out_node_off;
    v.tile_off = p.ws.tile_off;
    v.n_tiles = p.ws.hdr->n_tiles;
    v.ok = p.ws.hdr->ok;
  }
  const u32 b = blockIdx.x;
  if (b < nb_tiles) prep_tiles_block(p, v, b, s_lo);
  else if (b < nb_tiles + nb_patch) prep_patch(p, v, (u64)(b - nb_tiles) * 256 + threadIdx.x);
  else write_dims(p, v, (u64)(b - nb_tiles - nb_patch) * 256 + threadIdx.x);
}

bool desc_ok(const fdy_mat_desc* d) {
  if (!d) return false;
  if (d->n_graphs > (1u << 20) || d->n_src_graphs > (1u << 20) || d->n_templates > (1u << 20))
    return false;
  if (d->n_maps > 65535u) return false;
  if (d->out_words_per_map >= (1ull << 40)) return false;
  return true;
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t layout(const fdy_mat_desc* d, unsigned char* base, MatWs* ws) {
  const u64 max_tiles = (d->out_words_per_map + kMatTile - 1) / kMatTile + d->n_graphs;
  const u32 R = d->map_rank ? d->n_ranks : 0;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    unsigned char* p = base ? base + off : nullptr;
    off += align256(bytes);
    return p;
  };
  MatWs w;
  w.hdr = (MatHeader*)take(sizeof(MatHeader));
  w.out_word_off = (u64*)take(((size_t)d->n_graphs + 1) * 8);
  w.out_node_off = (u64*)take(((size_t)d->n_graphs + 1) * 8);
  w.tile_off = (u64*)take(((size_t)d->n_graphs + 1) * 8);
  w.tiles = (MatTile*)take((size_t)max_tiles * sizeof(MatTile));
  w.tile_patch = (uint2*)take((size_t)max_tiles * R * sizeof(uint2));
  w.max_tiles = (u32)max_tiles;
  if (ws) *ws = w;
  return off;
}

}  // namespace
}  // namespace fdy

using namespace fdy;

extern "C" size_t fdy_materialize_workspace_bytes(const fdy_mat_desc* h_desc) {
  if (!desc_ok(h_desc)) return 0;
  return layout(h_desc, nullptr, nullptr);
}

// Scratch of the entry point that allocates nothing (fdy_materialize_static): the tile table and
// the other per-call tables of a materialization, in device memory that belongs to the loaded
// library.  Each GPU holds its own copy at its own address, found once per device with
// hipGetSymbolAddress; host code uses that address, never the array's name.
constexpr size_t kStaticScratchBytes = 4u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static int materialize_launch(const fdy_mat_desc* h_desc, uint64_t* d_out_words, uint32_t* d_out_dims,
                              void* d_workspace, size_t workspace_bytes, uint32_t* d_status,
                              void* hip_stream);

extern "C" int fdy_materialize(const fdy_mat_desc* h_desc, uint64_t* d_out_words, uint32_t* d_out_dims,
                               void* d_workspace, size_t workspace_bytes, uint32_t* d_status,
                               void* hip_stream) {
  return materialize_launch(h_desc, d_out_words, d_out_dims, d_workspace, workspace_bytes, d_status, hip_stream);
}

extern "C" size_t fdy_materialize_static_limit(void) { return kStaticScratchBytes; }

extern "C" int fdy_materialize_static(const fdy_mat_desc* h_desc, uint64_t* d_out_words, uint32_t* d_out_dims,
                                      uint32_t* d_status, void* hip_stream) {
  if (!desc_ok(h_desc)) return FDY_ERR_INVALID_ARG;
  if (layout(h_desc, nullptr, nullptr) > kStaticScratchBytes) return FDY_ERR_WORKSPACE;  // beyond the fixed scratch
  constexpr int kMaxDevices = 64;
  static void* ptr_of_device[kMaxDevices] = {};
  static std::mutex mu;
  int dev = 0;
  FDY_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return FDY_ERR_INVALID_ARG;
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of_device[dev]) {  // first call on this device, which is current
      void* found = nullptr;
      FDY_HIP_TRY(hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)));
      if (!found) return FDY_ERR_HIP;
      ptr_of_device[dev] = found;
    }
    ptr = ptr_of_device[dev];
  }
  return materialize_launch(h_desc, d_out_words, d_out_dims, ptr, kStaticScratchBytes, d_status, hip_stream);
}

static int materialize_launch(const fdy_mat_desc* h_desc, uint64_t* d_out_words, uint32_t* d_out_dims,
                              void* d_workspace, size_t workspace_bytes, uint32_t* d_status,
                              void* hip_stream) {
  if (!desc_ok(h_desc)) return FDY_ERR_INVALID_ARG;
  const fdy_mat_desc& d = *h_desc;
  if (d.n_graphs == 0 || d.n_maps == 0) return FDY_OK;
  if (!d.src_word_off || !d.src_reloc_off || !d.tmpl_graph || !d.graph_tmpl || !d.ovr_off ||
      !d.new_base)
    return FDY_ERR_INVALID_ARG;
  if (d.out_words_per_map && (!d_out_words || ((uintptr_t)d_out_words & 15) || !d.src_words ||
                              ((uintptr_t)d.src_words & 15)))
    return FDY_ERR_INVALID_ARG;
  if ((uintptr_t)d.relocs & 15 || (uintptr_t)d.patch & 15) return FDY_ERR_INVALID_ARG;
  if (d.map_rank && (d.n_ranks == 0 || !d.patch_off)) return FDY_ERR_INVALID_ARG;
  if (d_out_dims && (((uintptr_t)d_out_dims & 7) || !d.src_node_off || !d.govr_off ||
                     (d.out_nodes_total && !d.src_nodes)))
    return FDY_ERR_INVALID_ARG;
  MatParams p;
  p.d = d;
  if (!d.map_rank) p.d.n_ranks = 0;
  if (!d_out_dims) p.d.out_nodes_total = 0;
  const size_t need = layout(&d, nullptr, nullptr);
  if (!d_workspace || ((uintptr_t)d_workspace & 255) || workspace_bytes < need) return FDY_ERR_WORKSPACE;
  layout(&d, (unsigned char*)d_workspace, &p.ws);
  p.out_words = (u64*)d_out_words;
  p.out_dims = d_out_dims;
  p.d_status = d_status;
  p.map_group = 1;
  hipStream_t stream = (hipStream_t)hip_stream;
  (void)hipGetLastError();  // drop any stale error left by earlier, unrelated runtime calls

  // Base maps per workgroup.  Measured on MI355X, groups above 2 (4 with rank patches) lose
  // more to the coarser tail of the launch than they save in repeated loads.
  u32 mg = (u32)fdy__tune_get(FDY_TUNE_MAT_MAP_GROUP);
  if (mg == 0) mg = d.map_rank ? 4 : 2;
  p.map_group = mg < d.n_maps ? mg : d.n_maps;
  const u32 n_groups = (d.n_maps + p.map_group - 1) / p.map_group;
  p.stream_once = n_groups == 1 && p.ws.max_tiles >= (u32)fdy__tune_get(FDY_TUNE_MAT_ONCE_TILES) ? 1u : 0u;
  const u32 nb_dims_all = (d_out_dims && d.out_nodes_total) ? (u32)((d.out_nodes_total + 255) / 256) : 0;
  // A launch small enough that all its workgroups run side by side resolves its tiles itself.
  const u64 self_limit = (u64)fdy__tune_get(FDY_TUNE_MAT_SELF_WGS);
  if (d.n_graphs <= kSelfGraphs && p.map_group <= kSelfMaxGroup && p.ws.max_tiles &&
      (u64)p.ws.max_tiles * n_groups <= self_limit) {
    launch(FDY_PROF_MAT_MAIN, mat_main_kernel<true>, dim3(p.ws.max_tiles + nb_dims_all + kCheckBlocks, n_groups),
           dim3(kMatBlock), 0, stream, p, p.ws.max_tiles, nb_dims_all);
    FDY_HIP_TRY(hipGetLastError());
    return FDY_OK;
  }

  const bool own_sums = d.n_graphs <= kOwnSumsMax;
  if (!own_sums) {
    launch(FDY_PROF_MAT_PREP_GRAPHS, mat_prep_graphs_kernel, dim3(1), dim3(1024), 0, stream, p);
    FDY_HIP_TRY(hipGetLastError());
  }
  u32 nb_tiles = (p.ws.max_tiles + kPrepTiles - 1) / kPrepTiles;
  const u32 nb_patch = p.d.map_rank ? (u32)(((u64)p.ws.max_tiles * p.d.n_ranks + 255) / 256) : 0;
  const u32 nb_dims = (d_out_dims && d.out_nodes_total) ? (u32)((d.out_nodes_total + 255) / 256) : 0;
  if (own_sums && nb_tiles + nb_patch + nb_dims == 0) nb_tiles = 1;  // someone has to verify the totals
  if (nb_tiles + nb_patch + nb_dims) {
    const u32 nb = nb_tiles + nb_patch + nb_dims + kCheckBlocks;
    launch(FDY_PROF_MAT_PREP_TILES, own_sums ? mat_prep_tiles_kernel<true> : mat_prep_tiles_kernel<false>, dim3(nb),
           dim3(256), 0, stream, p, nb_tiles, nb_patch);
    FDY_HIP_TRY(hipGetLastError());
  }
  if (p.ws.max_tiles) {
    launch(FDY_PROF_MAT_MAIN, mat_main_kernel<false>, dim3(p.ws.max_tiles, n_groups), dim3(kMatBlock), 0, stream, p,
           p.ws.max_tiles, 0u);
    FDY_HIP_TRY(hipGetLastError());
  }
  return FDY_OK;
}
