// fdy_oracle.cpp - the CPU oracle.  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// A plain, single-threaded, obviously-correct C++17 statement of what the three data
// transforms compute.  It exists so that the HIP library can be checked bit for bit; it
// shares no source, header, table or helper with the HIP path and must never be imported,
// linked or called by it (only tests, the smoke check and the bench's cpu_baseline leg do).
//
// What each function follows:
//  * scan          - the paper does not scan (Section 4.1.1 makes every captured address
//                    valid again by forcing an identical layout).  The definition used here
//                    is the relaxation this repository targets: a word is a pointer iff it
//                    lies in one of the half-open ranges of the allocation table that the
//                    deterministic allocator records (Section 4.1.1, Section 5.1).  It has
//                    a plain definition, written out below with std::upper_bound, and a
//                    second, linear-search form for pinning.
//  * fingerprint   - Section 4.2.1 / Section 5.3 ("a key based on topology", graphs with
//                    identical keys are grouped).  The paper fixes no key function; the
//                    one written here (SplitMix64 output function + polynomial fold) is
//                    this repository's reading.  Exact grouping by record equality and a
//                    closed-form power-sum evaluation are provided for pinning.
//  * materialize   - Section 4.2.1 (prepare the parameter sets of non-template graphs from
//                    the template) and Section 4.2.2 (patch rank-specific communication
//                    arguments): copy, rebase, override, patch, in that order.  A
//                    word-at-a-time form is provided for pinning.
//
//  * derive        - the SAVE side of Section 4.2.1 / Section 5.3: within a topology group
//                    the graphs "differ only in per-node parameters", so a non-template graph
//                    is stored as what differs from its template.  The plain definition: every
//                    32-bit half of the graph's argument words that is not equal to the
//                    template's half at the same place, in ascending byte order.
//
// Parity pins (see tests/test_oracle_*.py): brute-force forms on small inputs, generator
// ground truth (every planted pointer found, no boundary decoy flagged), identity and
// round-trip invariants, the published SplitMix64 test vector.  No function here is
// "parity unpinned".
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

struct Alloc { uint64_t base, size; };
struct Node { uint64_t kernel_id; uint32_t grid[3]; uint32_t block[3]; uint32_t blob_len; uint32_t flags; };
struct Reloc { uint32_t word, region; uint64_t offset; };
struct Ovr32 { uint32_t byte_off, value; };
struct GridOvr { uint32_t node; uint32_t grid[3]; };
struct Patch { uint32_t word, reserved; uint64_t value; };

static_assert(sizeof(Alloc) == 16 && sizeof(Node) == 40 && sizeof(Reloc) == 16, "layout");
static_assert(sizeof(Ovr32) == 8 && sizeof(GridOvr) == 16 && sizeof(Patch) == 16, "layout");

constexpr uint64_t kP = 0x9e3779b97f4a7c15ull;

uint64_t mix(uint64_t x) {
  x ^= x >> 30; x *= 0xbf58476d1ce4e5b9ull;
  x ^= x >> 27; x *= 0x94d049bb133111ebull;
  x ^= x >> 31;
  return x;
}

// field-mask bits
enum : uint32_t { KID = 1, GX = 2, GY = 4, GZ = 8, BLK = 16, LEN = 32, FLG = 64 };

Node masked(const Node& n, uint32_t mask) {
  Node m;
  std::memset(&m, 0, sizeof m);
  if (mask & KID) m.kernel_id = n.kernel_id;
  if (mask & GX) m.grid[0] = n.grid[0];
  if (mask & GY) m.grid[1] = n.grid[1];
  if (mask & GZ) m.grid[2] = n.grid[2];
  if (mask & BLK) { m.block[0] = n.block[0]; m.block[1] = n.block[1]; m.block[2] = n.block[2]; }
  if (mask & LEN) m.blob_len = n.blob_len;
  if (mask & FLG) m.flags = n.flags;
  return m;
}

uint64_t node_hash(const Node& raw, uint32_t mask) {
  const Node n = masked(raw, mask);
  uint64_t a = mix(n.kernel_id + kP);
  a = mix(a ^ ((uint64_t)n.grid[0] | ((uint64_t)n.grid[1] << 32)));
  a = mix(a ^ ((uint64_t)n.grid[2] | ((uint64_t)n.block[0] << 32)));
  a = mix(a ^ ((uint64_t)n.block[1] | ((uint64_t)n.block[2] << 32)));
  a = mix(a ^ ((uint64_t)n.blob_len | ((uint64_t)n.flags << 32)));
  return a;
}

void dense_ids_by_first_appearance(const std::vector<uint32_t>& first, uint32_t G,
                                   uint32_t* template_id, uint32_t* tmpl_graph, uint32_t* n_templates) {
  uint32_t T = 0;
  for (uint32_t g = 0; g < G; ++g) {
    if (first[g] == g) {
      if (tmpl_graph) tmpl_graph[T] = g;
      template_id[g] = T++;
    } else {
      template_id[g] = template_id[first[g]];
    }
  }
  *n_templates = T;
}

}  // namespace

extern "C" {

uint64_t orc_mix(uint64_t x) { return mix(x); }

// Table rules: strictly ascending base, size >= 1, base+size does not wrap, no overlap
// (touching allowed).  Returns 0 if valid, else -2 with *bad = first offending entry.
int orc_table_validate(const Alloc* t, uint32_t n, uint32_t* bad) {
  for (uint32_t i = 0; i < n; ++i) {
    bool ok = t[i].size >= 1 && t[i].base + t[i].size > t[i].base;
    if (ok && i > 0) ok = t[i - 1].base < t[i].base && t[i - 1].base + t[i - 1].size <= t[i].base;
    if (!ok) { if (bad) *bad = i; return -2; }
  }
  return 0;
}

// Scan: for every word in ascending order, i = (number of bases <= w) - 1; hit iff i >= 0
// and w - base[i] < size[i].  Writes at most `capacity` entries; *count = all hits.
int orc_scan(const uint64_t* words, uint64_t n_words, const Alloc* table, uint32_t n_alloc,
             Reloc* relocs, uint64_t capacity, uint64_t* count) {
  std::vector<uint64_t> bases(n_alloc);
  for (uint32_t i = 0; i < n_alloc; ++i) bases[i] = table[i].base;
  uint64_t K = 0;
  for (uint64_t j = 0; j < n_words; ++j) {
    const uint64_t w = words[j];
    const int64_t i = (std::upper_bound(bases.begin(), bases.end(), w) - bases.begin()) - 1;
    if (i >= 0 && (w - table[i].base) < table[i].size) {
      if (K < capacity) relocs[K] = Reloc{(uint32_t)j, (uint32_t)i, w - table[i].base};
      ++K;
    }
  }
  *count = K;
  return 0;
}

// The same relation by linear search over every interval, highest index wins (for a valid
// table at most one interval matches).  For pinning orc_scan on small inputs.
int orc_scan_brute(const uint64_t* words, uint64_t n_words, const Alloc* table, uint32_t n_alloc,
                   Reloc* relocs, uint64_t capacity, uint64_t* count) {
  uint64_t K = 0;
  for (uint64_t j = 0; j < n_words; ++j) {
    const uint64_t w = words[j];
    int64_t hit = -1;
    for (uint32_t i = 0; i < n_alloc; ++i)
      if (w >= table[i].base && w - table[i].base < table[i].size) hit = i;
    if (hit >= 0) {
      if (K < capacity) relocs[K] = Reloc{(uint32_t)j, (uint32_t)hit, w - table[hit].base};
      ++K;
    }
  }
  *count = K;
  return 0;
}

// Scan at 4-byte stride (variant for pointers at 4-byte alignment; argument buffers are
// opaque bytes, Section 2.2 / Appendix B): the array is n_units 32-bit little-endian units,
// position q in [0, n_units - 1) is the value unit[q] + 2^32 * unit[q + 1], classified as in
// orc_scan; reloc.word = q.  The values are written out one by one and handed to orc_scan.
int orc_scan_stride4(const uint32_t* units, uint64_t n_units, const Alloc* table, uint32_t n_alloc,
                     Reloc* relocs, uint64_t capacity, uint64_t* count) {
  std::vector<uint64_t> value(n_units ? n_units - 1 : 0);
  for (uint64_t q = 0; q + 1 < n_units; ++q) value[q] = (uint64_t)units[q] | ((uint64_t)units[q + 1] << 32);
  return orc_scan(value.data(), value.size(), table, n_alloc, relocs, capacity, count);
}

// out[s] = number of relocs (of the first n_relocs) with word < word_off[s].
int orc_reloc_segment(const Reloc* relocs, uint64_t n_relocs, const uint64_t* word_off,
                      uint32_t n_off, uint64_t* out) {
  for (uint32_t s = 0; s < n_off; ++s) {
    uint64_t c = 0;
    while (c < n_relocs && (uint64_t)relocs[c].word < word_off[s]) ++c;
    out[s] = c;
  }
  return 0;
}

// key(g) by Horner's rule, then dense template ids in order of first appearance.
int orc_fingerprint(const Node* nodes, const uint64_t* node_off, uint32_t G, uint32_t mask,
                    uint64_t* keys, uint32_t* template_id, uint32_t* tmpl_graph, uint32_t* n_templates) {
  for (uint32_t g = 0; g < G; ++g) {
    const uint64_t N = node_off[g + 1] - node_off[g];
    uint64_t H = mix(N);
    for (uint64_t n = 0; n < N; ++n) H = H * kP + node_hash(nodes[node_off[g] + n], mask);
    keys[g] = mix(H);
  }
  std::vector<uint32_t> first(G);
  for (uint32_t g = 0; g < G; ++g) {
    first[g] = g;
    for (uint32_t h = 0; h < g; ++h)
      if (keys[h] == keys[g]) { first[g] = h; break; }
  }
  dense_ids_by_first_appearance(first, G, template_id, tmpl_graph, n_templates);
  return 0;
}

// Second evaluation of the key for pinning: mix( mix(N)*P^N + sum_n h_n * P^(N-1-n) ),
// with the powers built by repeated multiplication from the last node backwards.
int orc_fingerprint_powersum(const Node* nodes, const uint64_t* node_off, uint32_t G, uint32_t mask,
                             uint64_t* keys) {
  for (uint32_t g = 0; g < G; ++g) {
    const uint64_t N = node_off[g + 1] - node_off[g];
    uint64_t sum = 0, pw = 1;
    for (uint64_t n = N; n-- > 0;) {
      sum += node_hash(nodes[node_off[g] + n], mask) * pw;
      pw *= kP;
    }
    keys[g] = mix(mix(N) * pw + sum);
  }
  return 0;
}

// Grouping by exact equality of the masked node sequences (no hashing).  For pinning the
// fingerprint grouping.
int orc_group_exact(const Node* nodes, const uint64_t* node_off, uint32_t G, uint32_t mask,
                    uint32_t* template_id, uint32_t* tmpl_graph, uint32_t* n_templates) {
  auto same = [&](uint32_t a, uint32_t b) {
    const uint64_t Na = node_off[a + 1] - node_off[a], Nb = node_off[b + 1] - node_off[b];
    if (Na != Nb) return false;
    for (uint64_t n = 0; n < Na; ++n) {
      const Node x = masked(nodes[node_off[a] + n], mask), y = masked(nodes[node_off[b] + n], mask);
      if (std::memcmp(&x, &y, sizeof x) != 0) return false;
    }
    return true;
  };
  std::vector<uint32_t> first(G);
  for (uint32_t g = 0; g < G; ++g) {
    first[g] = g;
    for (uint32_t h = 0; h < g; ++h)
      if (first[h] == h && same(h, g)) { first[g] = h; break; }
  }
  dense_ids_by_first_appearance(first, G, template_id, tmpl_graph, n_templates);
  return 0;
}

struct MatArgs {
  uint32_t S, T, G, M, A, R;
  const uint64_t* src_words; const uint64_t* src_word_off;
  const Node* src_nodes; const uint64_t* src_node_off;
  const Reloc* relocs; const uint64_t* src_reloc_off;
  const uint32_t* tmpl_graph; const uint32_t* graph_tmpl;
  const Ovr32* ovr; const uint64_t* ovr_off;
  const GridOvr* govr; const uint64_t* govr_off;
  const uint64_t* new_base; const uint32_t* map_rank;
  const Patch* patch; const uint64_t* patch_off;
};

// Checks every index the transform dereferences.  0 = usable, -1 = not.
int orc_materialize_validate(const MatArgs* a, uint64_t out_words_per_map, uint64_t out_nodes_total) {
  uint64_t words = 0, nnodes = 0;
  for (uint32_t t = 0; t < a->T; ++t) {
    const uint32_t s = a->tmpl_graph[t];
    if (s >= a->S) return -1;
    const uint64_t w0 = a->src_word_off[s], w1 = a->src_word_off[s + 1];
    for (uint64_t k = a->src_reloc_off[s]; k < a->src_reloc_off[s + 1]; ++k) {
      if (a->relocs[k].word < w0 || a->relocs[k].word >= w1 || a->relocs[k].region >= a->A) return -1;
      if (k > a->src_reloc_off[s] && a->relocs[k - 1].word >= a->relocs[k].word) return -1;
    }
    for (uint32_t r = 0; r < a->R; ++r)
      for (uint64_t k = a->patch_off[t * a->R + r]; k < a->patch_off[t * a->R + r + 1]; ++k) {
        if (a->patch[k].word >= w1 - w0) return -1;
        if (k > a->patch_off[t * a->R + r] && a->patch[k - 1].word >= a->patch[k].word) return -1;
      }
  }
  for (uint32_t g = 0; g < a->G; ++g) {
    const uint32_t t = a->graph_tmpl[g];
    if (t >= a->T) return -1;
    const uint32_t s = a->tmpl_graph[t];
    const uint64_t nw = a->src_word_off[s + 1] - a->src_word_off[s];
    const uint64_t nn = a->src_node_off ? a->src_node_off[s + 1] - a->src_node_off[s] : 0;
    for (uint64_t k = a->ovr_off[g]; k < a->ovr_off[g + 1]; ++k) {
      if (a->ovr[k].byte_off % 4 != 0 || (uint64_t)a->ovr[k].byte_off + 4 > nw * 8) return -1;
      if (k > a->ovr_off[g] && a->ovr[k - 1].byte_off >= a->ovr[k].byte_off) return -1;
    }
    for (uint64_t k = a->govr_off[g]; k < a->govr_off[g + 1]; ++k) {
      if (a->govr[k].node >= nn) return -1;
      if (k > a->govr_off[g] && a->govr[k - 1].node >= a->govr[k].node) return -1;
    }
    words += nw;
    nnodes += nn;
  }
  if (a->map_rank)
    for (uint32_t m = 0; m < a->M; ++m)
      if (a->map_rank[m] >= a->R) return -1;
  if (words != out_words_per_map) return -1;
  if (out_nodes_total != 0 && nnodes != out_nodes_total) return -1;
  return 0;
}

// Materialize, stage by stage in the fixed order copy -> rebase -> override -> patch.
// out_words is [M][out_words_per_map]; out_dims is [out_nodes_total][6] or NULL.
int orc_materialize(const MatArgs* a, uint64_t* out_words, uint64_t out_words_per_map,
                    uint32_t* out_dims, uint64_t out_nodes_total) {
  if (orc_materialize_validate(a, out_words_per_map, out_dims ? out_nodes_total : 0) != 0) return -1;
  for (uint32_t m = 0; m < a->M; ++m) {
    uint64_t* out = out_words + (uint64_t)m * out_words_per_map;
    for (uint32_t g = 0; g < a->G; ++g) {
      const uint32_t t = a->graph_tmpl[g];
      const uint32_t s = a->tmpl_graph[t];
      const uint64_t w0 = a->src_word_off[s];
      const uint64_t nw = a->src_word_off[s + 1] - w0;
      // c1: copy the template blob
      for (uint64_t k = 0; k < nw; ++k) out[k] = a->src_words[w0 + k];
      // c2: rebase every relocated word
      for (uint64_t k = a->src_reloc_off[s]; k < a->src_reloc_off[s + 1]; ++k) {
        const Reloc& r = a->relocs[k];
        out[r.word - w0] = a->new_base[(uint64_t)m * a->A + r.region] + r.offset;
      }
      // c3: per-graph 32-bit scalar overrides (little-endian store into the blob bytes)
      for (uint64_t k = a->ovr_off[g]; k < a->ovr_off[g + 1]; ++k) {
        const uint32_t v = a->ovr[k].value;
        std::memcpy(reinterpret_cast<unsigned char*>(out) + a->ovr[k].byte_off, &v, 4);
      }
      // c4: rank-dependent whole-word patches
      if (a->map_rank) {
        const uint64_t row = (uint64_t)t * a->R + a->map_rank[m];
        for (uint64_t k = a->patch_off[row]; k < a->patch_off[row + 1]; ++k)
          out[a->patch[k].word] = a->patch[k].value;
      }
      out += nw;
    }
  }
  if (out_dims) {
    uint32_t* d = out_dims;
    for (uint32_t g = 0; g < a->G; ++g) {
      const uint32_t s = a->tmpl_graph[a->graph_tmpl[g]];
      const uint64_t n0 = a->src_node_off[s], nn = a->src_node_off[s + 1] - n0;
      for (uint64_t n = 0; n < nn; ++n) {
        const Node& nd = a->src_nodes[n0 + n];
        for (int c = 0; c < 3; ++c) { d[n * 6 + c] = nd.grid[c]; d[n * 6 + 3 + c] = nd.block[c]; }
      }
      for (uint64_t k = a->govr_off[g]; k < a->govr_off[g + 1]; ++k)
        for (int c = 0; c < 3; ++c) d[(uint64_t)a->govr[k].node * 6 + c] = a->govr[k].grid[c];
      d += nn * 6;
    }
  }
  return 0;
}

// The same result one output word at a time: every list is searched linearly for entries
// that touch this word, and the stages are applied to that single word in order.  For
// pinning orc_materialize on small inputs.
int orc_materialize_brute(const MatArgs* a, uint64_t* out_words, uint64_t out_words_per_map) {
  if (orc_materialize_validate(a, out_words_per_map, 0) != 0) return -1;
  for (uint32_t m = 0; m < a->M; ++m) {
    uint64_t pos = 0;
    for (uint32_t g = 0; g < a->G; ++g) {
      const uint32_t t = a->graph_tmpl[g];
      const uint32_t s = a->tmpl_graph[t];
      const uint64_t w0 = a->src_word_off[s];
      const uint64_t nw = a->src_word_off[s + 1] - w0;
      for (uint64_t k = 0; k < nw; ++k) {
        uint64_t v = a->src_words[w0 + k];
        for (uint64_t q = a->src_reloc_off[s]; q < a->src_reloc_off[s + 1]; ++q)
          if (a->relocs[q].word == w0 + k)
            v = a->new_base[(uint64_t)m * a->A + a->relocs[q].region] + a->relocs[q].offset;
        for (uint64_t q = a->ovr_off[g]; q < a->ovr_off[g + 1]; ++q) {
          if (a->ovr[q].byte_off / 8 != k) continue;
          if (a->ovr[q].byte_off % 8 == 0) v = (v & 0xffffffff00000000ull) | a->ovr[q].value;
          else v = (v & 0x00000000ffffffffull) | ((uint64_t)a->ovr[q].value << 32);
        }
        if (a->map_rank) {
          const uint64_t row = (uint64_t)t * a->R + a->map_rank[m];
          for (uint64_t q = a->patch_off[row]; q < a->patch_off[row + 1]; ++q)
            if (a->patch[q].word == k) v = a->patch[q].value;
        }
        out_words[(uint64_t)m * out_words_per_map + pos + k] = v;
      }
      pos += nw;
    }
  }
  return 0;
}

// Per-graph overrides by comparison with the template: for graph g, template source graph
// s = tmpl_graph[graph_tmpl[g]], every byte offset b (multiple of 4) at which the 32-bit
// little-endian value of g's blob differs from s's becomes {b, value in g}; ascending b per
// graph, graphs in order; ovr_off[g] = entries before graph g, ovr_off[G] = total (also when
// it exceeds `capacity`; then only the first `capacity` entries are stored).
// -1: a template index out of range, a graph whose word count differs from its template's,
// or a graph of 2^29 words or more.
int orc_derive_overrides(const uint64_t* words, const uint64_t* word_off, uint32_t G,
                         const uint32_t* graph_tmpl, const uint32_t* tmpl_graph, uint32_t T, Ovr32* ovr,
                         uint64_t capacity, uint64_t* ovr_off) {
  uint64_t K = 0;
  for (uint32_t g = 0; g < G; ++g) {
    ovr_off[g] = K;
    if (graph_tmpl[g] >= T) return -1;
    const uint32_t s = tmpl_graph[graph_tmpl[g]];
    if (s >= G) return -1;
    const uint64_t nw = word_off[g + 1] - word_off[g];
    if (word_off[s + 1] - word_off[s] != nw) return -1;
    if (nw >> 29) return -1;  // byte offsets are 32-bit
    const unsigned char* a = reinterpret_cast<const unsigned char*>(words + word_off[g]);
    const unsigned char* b = reinterpret_cast<const unsigned char*>(words + word_off[s]);
    for (uint64_t off = 0; off < nw * 8; off += 4) {
      uint32_t va, vb;
      std::memcpy(&va, a + off, 4);
      std::memcpy(&vb, b + off, 4);
      if (va != vb) {
        if (K < capacity) {
          ovr[K].byte_off = (uint32_t)off;
          ovr[K].value = va;
        }
        ++K;
      }
    }
  }
  ovr_off[G] = K;
  return 0;
}

}  // extern "C"
