// install_scale.hip - hipGraph install at the scale of a decode graph (test program, not part
// of the library).
//
// Section 4.2.1 / Section 5.3 and Table 2 of the paper: one template graph is instantiated per
// unique topology; a target graph is brought up by applying its node parameters (kernel
// arguments and launch dimensions) to the executable graph of ITS template, in place, which
// the paper times per graph against building and instantiating the graph from scratch.
// This program does the same with parameters produced by libfdy, at the node count of one
// dense-decode graph and with three topologies side by side:
//   1. `n_graphs` graphs are "captured" on buffer set A (one slab; node i of every graph reads
//      buffer i and writes buffer i + 1).  They fall into three topology buckets by graph
//      number (as the batch sizes of a model do); the buckets differ in which nodes run the
//      second toy kernel.  Inside a bucket the graphs differ in two 32-bit scalars and in the
//      grid.x of the two nodes that take them;
//   2. the archive (every graph's argument words and node records) is scanned against set A's
//      allocation table, segmented, fingerprinted with grid.x masked out (three templates must
//      come out), the scalar overrides are derived on the device (fdy_derive_overrides), and
//      everything is materialized for `n_maps` other slabs, launch dimensions included (grid
//      overrides from the graphs' node records);
//   3. one template hipGraph per topology is built from the words of the graph that the
//      fingerprint named as its template, and instantiated once;
//   4. for every (map, graph) the materialized words (copied to the host once per map) and
//      launch dimensions are installed node by node with hipGraphExecKernelNodeSetParams into
//      the executable graph of the graph's template; the install is timed on the host clock;
//      the graph is launched and the last buffer of the map's slab is compared with a host
//      simulation of the chain, which depends on every node's kernel, scalar and gridDim.x;
//      set A must stay untouched;
//   5. for comparison, building and instantiating a fresh graph of the same nodes is timed.
// Results go to `stats`: [0] install ms per graph (median), [1] min, [2] max, [3] build +
// instantiate ms per graph (median of 5), [4] launch + sync ms per graph (median), [5] number of
// (map, graph) pairs verified, [6] relocations found, [7] device-to-host copy ms per map,
// [8] ms per graph of the whole-graph form of the update (set the parameters on the graph's nodes,
// then one hipGraphExecUpdate; median over up to eight graphs), [9] templates found, [10]
// executable graphs that received at least one install, [11] installs that set a gridDim.x
// other than the template's.  `stats` holds 12 doubles.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <vector>

#include "fdy.h"

namespace {

constexpr uint32_t kElems = 64;            // elements per buffer (512 bytes)
constexpr uint64_t kBufBytes = kElems * 8;
constexpr uint64_t kStride = 1024;         // buffers sit 1 KiB apart inside a slab
constexpr uint32_t kTopologies = 3;

// Both kernels fold gridDim.x into the result: an install that sets the wrong grid fails the
// comparison with the host simulation.  Only block 0 has elements to write.
__global__ void chain_kernel(const uint64_t* src, uint64_t* dst, uint32_t k, uint32_t n) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i] * k + i + 1000ull * gridDim.x;
}
__global__ void chain_kernel_b(const uint64_t* src, uint64_t* dst, uint32_t k, uint32_t n) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = (src[i] ^ k) + 3ull * i + 1000ull * gridDim.x;
}
uint64_t step_value(bool b, uint64_t x, uint32_t k, uint32_t i, uint32_t gx) {
  return b ? (x ^ k) + 3ull * i + 1000ull * gx : x * k + i + 1000ull * gx;
}

struct Args {  // the argument buffer of one node as a serializer would record it
  uint64_t src, dst;
  uint32_t k, n;
};
static_assert(sizeof(Args) == 24, "three 8-byte words");

#define CK(expr)                                                                  \
  do {                                                                            \
    hipError_t e__ = (expr);                                                      \
    if (e__ != hipSuccess) {                                                      \
      snprintf(msg, msg_len, "%s failed: %s", #expr, hipGetErrorString(e__));     \
      return 1;                                                                   \
    }                                                                             \
  } while (0)
#define FD(expr)                                                                  \
  do {                                                                            \
    int r__ = (expr);                                                             \
    if (r__ != FDY_OK) {                                                          \
      snprintf(msg, msg_len, "%s failed: %s", #expr, fdy_strerror(r__));          \
      return 1;                                                                   \
    }                                                                             \
  } while (0)

template <typename T>
struct DevBuf {
  T* p = nullptr;
  ~DevBuf() { if (p) (void)hipFree(p); }
  hipError_t alloc(size_t n) { return hipMalloc((void**)&p, n * sizeof(T) ? n * sizeof(T) : 1); }
  template <typename V>
  hipError_t upload(const V& v) {
    hipError_t e = alloc(v.size());
    if (e != hipSuccess || v.empty()) return e;
    return hipMemcpy(p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice);
  }
};

double now_ms() {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

double median(std::vector<double> v) {
  std::sort(v.begin(), v.end());
  return v.empty() ? 0.0 : v[v.size() / 2];
}

// What the "capture" of graph g holds.
struct Shape {
  uint32_t n_nodes, n_graphs;
  uint32_t bucket(uint32_t g) const { return g < (n_graphs + 7) / 8 ? 0 : (g < (n_graphs + 1) / 2 ? 1 : 2); }
  bool uses_b(uint32_t t, uint32_t i) const { return i % 16 == 3 + 4 * t; }  // the second kernel
  uint32_t scalar_node(int which) const { return which ? (n_nodes / 2 + 1) % n_nodes : 2 % n_nodes; }
  bool takes_scalar(uint32_t i) const { return i == scalar_node(0) || i == scalar_node(1); }
  uint32_t k(uint32_t g, uint32_t i) const {  // the node's scalar argument in graph g
    if (i == scalar_node(1)) return 101 + 2 * g;
    if (i == scalar_node(0)) return 100 + 2 * g;
    return 2 + i % 5;
  }
  uint32_t grid_x(uint32_t g, uint32_t i) const { return takes_scalar(i) ? 1 + g % 4 : 1; }
};

void fill_node_params(hipKernelNodeParams* np, void** params, Args* a, bool b, uint32_t gx, uint32_t gy, uint32_t gz,
                      uint32_t bx, uint32_t by, uint32_t bz) {
  params[0] = &a->src;
  params[1] = &a->dst;
  params[2] = &a->k;
  params[3] = &a->n;
  memset(np, 0, sizeof *np);
  np->func = b ? (void*)chain_kernel_b : (void*)chain_kernel;
  np->gridDim = dim3(gx, gy, gz);
  np->blockDim = dim3(bx, by, bz);
  np->kernelParams = params;
}

}  // namespace

extern "C" int install_scale_check(uint32_t n_nodes, uint32_t n_graphs, uint32_t n_maps, double* stats,
                                   char* msg, int msg_len) {
  if (n_nodes < 16 || n_nodes > 4096 || n_graphs < 8 || n_graphs > 512 || n_maps < 1 || n_maps > 8) {
    snprintf(msg, msg_len, "sizes out of range");
    return 1;
  }
  const Shape sh{n_nodes, n_graphs};
  hipStream_t stream;
  CK(hipStreamCreate(&stream));
  const uint32_t n_buf = n_nodes + 1;
  const size_t slab_bytes = (size_t)n_buf * kStride;
  // slab 0 is set A (the captured layout), slabs 1..n_maps are the new layouts
  std::vector<DevBuf<unsigned char>> slab(n_maps + 1);
  std::vector<uint64_t> init(kElems);
  for (uint32_t i = 0; i < kElems; ++i) init[i] = 3 + i;
  for (uint32_t s = 0; s <= n_maps; ++s) {
    CK(slab[s].alloc(slab_bytes));
    CK(hipMemset(slab[s].p, 0xA5, slab_bytes));
    CK(hipMemcpy(slab[s].p, init.data(), kBufBytes, hipMemcpyHostToDevice));
  }
  auto buf_addr = [&](uint32_t s, uint32_t b) { return (uint64_t)(uintptr_t)slab[s].p + (uint64_t)b * kStride; };

  // 1. the archive: every graph's argument words and node records, as captured on set A
  const uint64_t words_per_graph = (uint64_t)n_nodes * 3, n_words = words_per_graph * n_graphs;
  std::vector<Args> captured((size_t)n_graphs * n_nodes);
  std::vector<fdy_node> recs((size_t)n_graphs * n_nodes);
  std::vector<uint64_t> word_off(n_graphs + 1), node_off(n_graphs + 1), govr_off(n_graphs + 1);
  for (uint32_t g = 0; g < n_graphs; ++g) {
    const uint32_t t = sh.bucket(g);
    word_off[g] = g * words_per_graph;
    node_off[g] = (uint64_t)g * n_nodes;
    for (uint32_t i = 0; i < n_nodes; ++i) {
      captured[(size_t)g * n_nodes + i] = Args{buf_addr(0, i), buf_addr(0, i + 1), sh.k(g, i), kElems};
      fdy_node& r = recs[(size_t)g * n_nodes + i];
      memset(&r, 0, sizeof r);
      r.kernel_id = 0x1000 + i % 16 + (sh.uses_b(t, i) ? 0x100 : 0);  // sixteen kernels per layer
      r.grid[0] = sh.grid_x(g, i);
      r.grid[1] = r.grid[2] = 1;
      r.block[0] = kElems;
      r.block[1] = r.block[2] = 1;
      r.blob_len = sizeof(Args);
    }
  }
  word_off[n_graphs] = n_words;
  node_off[n_graphs] = (uint64_t)n_graphs * n_nodes;

  // 2. scan, segment, fingerprint (grid.x is a per-graph parameter, not topology), derive the
  // scalar overrides, materialize words and launch dimensions
  std::vector<fdy_alloc> table(n_buf);
  for (uint32_t b = 0; b < n_buf; ++b) table[b] = fdy_alloc{buf_addr(0, b), kBufBytes};
  uint32_t bad = 0;
  FD(fdy_table_validate(table.data(), n_buf, &bad));
  std::vector<uint64_t> new_base((size_t)n_maps * n_buf);
  for (uint32_t m = 0; m < n_maps; ++m)
    for (uint32_t b = 0; b < n_buf; ++b) new_base[(size_t)m * n_buf + b] = buf_addr(m + 1, b);

  DevBuf<uint64_t> d_words, d_count, d_word_off, d_reloc_off, d_new_base, d_out, d_ovr_off, d_govr_off, d_node_off,
      d_keys;
  DevBuf<fdy_alloc> d_table;
  DevBuf<fdy_reloc> d_relocs;
  DevBuf<fdy_node> d_recs;
  DevBuf<uint32_t> d_status, d_tmpl_graph, d_graph_tmpl, d_n_tmpl, d_dims;
  DevBuf<fdy_ovr32> d_ovr;
  DevBuf<fdy_grid_ovr> d_govr;
  DevBuf<unsigned char> d_ws_scan, d_ws_mat, d_ws_derive, d_prepared;
  CK(d_words.alloc(n_words + 2));
  CK(hipMemcpy(d_words.p, captured.data(), n_words * 8, hipMemcpyHostToDevice));
  CK(d_table.upload(table));
  CK(d_relocs.alloc(n_words));
  CK(d_count.alloc(1));
  CK(d_status.alloc(1));
  CK(hipMemset(d_status.p, 0, 4));
  const size_t prep_bytes = fdy_scan_table_bytes(n_buf, n_words);
  CK(d_prepared.alloc(prep_bytes));
  FD(fdy_scan_table_prepare(d_table.p, n_buf, n_words, d_prepared.p, prep_bytes, stream));
  const size_t ws_scan = fdy_scan_staging_bytes(n_words);
  CK(d_ws_scan.alloc(ws_scan));
  FD(fdy_scan_pointers(d_words.p, n_words, d_table.p, n_buf, d_relocs.p, n_words, d_count.p, d_prepared.p,
                       d_ws_scan.p, ws_scan, d_status.p, stream));
  CK(d_word_off.upload(word_off));
  CK(d_reloc_off.alloc(n_graphs + 1));
  CK(d_recs.upload(recs));
  CK(d_node_off.upload(node_off));
  CK(d_keys.alloc(n_graphs));
  CK(d_graph_tmpl.alloc(n_graphs));
  CK(d_tmpl_graph.alloc(n_graphs));
  CK(d_n_tmpl.alloc(1));
  FD(fdy_segment_fingerprint(d_relocs.p, d_count.p, n_words, d_word_off.p, d_reloc_off.p, d_recs.p, d_node_off.p,
                             n_graphs, FDY_FP_ALL & ~FDY_FP_GRID_X, d_keys.p, d_graph_tmpl.p, d_tmpl_graph.p,
                             d_n_tmpl.p, d_prepared.p, nullptr, 0, stream));
  CK(hipStreamSynchronize(stream));
  uint32_t n_templates = 0, status = 0;
  uint64_t count = 0;
  CK(hipMemcpy(&n_templates, d_n_tmpl.p, 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(&count, d_count.p, 8, hipMemcpyDeviceToHost));
  if (n_templates != kTopologies || count != 2ull * n_nodes * n_graphs) {
    snprintf(msg, msg_len, "%u templates (want %u), %llu pointers (want %llu)", n_templates, kTopologies,
             (unsigned long long)count, 2ull * n_nodes * n_graphs);
    return 1;
  }
  std::vector<uint32_t> graph_tmpl(n_graphs), tmpl_graph(n_templates);
  CK(hipMemcpy(graph_tmpl.data(), d_graph_tmpl.p, n_graphs * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(tmpl_graph.data(), d_tmpl_graph.p, n_templates * 4, hipMemcpyDeviceToHost));
  for (uint32_t g = 0; g < n_graphs; ++g)
    if (graph_tmpl[g] >= n_templates || sh.bucket(tmpl_graph[graph_tmpl[g]]) != sh.bucket(g)) {
      snprintf(msg, msg_len, "graph %u was grouped with a graph of another topology", g);
      return 1;
    }
  // scalar overrides: what each graph's words change in its template's, found on the device
  const uint64_t ovr_cap = 4ull * n_graphs;
  CK(d_ovr.alloc(ovr_cap));
  CK(d_ovr_off.alloc(n_graphs + 1));
  const size_t ws_derive = fdy_derive_workspace_bytes(n_words, n_graphs);
  CK(d_ws_derive.alloc(ws_derive));
  FD(fdy_derive_overrides(d_words.p, n_words, d_word_off.p, n_graphs, d_graph_tmpl.p, d_tmpl_graph.p, n_templates,
                          d_ovr.p, ovr_cap, d_ovr_off.p, d_ws_derive.p, ws_derive, d_status.p, stream));
  // grid overrides: the launch dimensions of a graph's node records that differ from its template's
  std::vector<fdy_grid_ovr> govr;
  for (uint32_t g = 0; g < n_graphs; ++g) {
    govr_off[g] = govr.size();
    const uint32_t tg = tmpl_graph[graph_tmpl[g]];
    for (uint32_t i = 0; i < n_nodes; ++i)
      if (sh.grid_x(g, i) != sh.grid_x(tg, i)) govr.push_back(fdy_grid_ovr{i, {sh.grid_x(g, i), 1, 1}});
  }
  govr_off[n_graphs] = govr.size();
  CK(d_govr.upload(govr));
  CK(d_govr_off.upload(govr_off));
  CK(d_new_base.upload(new_base));
  const uint64_t out_words_per_map = n_words, out_nodes_total = (uint64_t)n_graphs * n_nodes;
  CK(d_out.alloc((size_t)out_words_per_map * n_maps + 2));
  CK(d_dims.alloc((size_t)out_nodes_total * 6));
  fdy_mat_desc d;
  memset(&d, 0, sizeof d);
  d.n_src_graphs = n_graphs;
  d.n_templates = n_templates;
  d.n_graphs = n_graphs;
  d.n_maps = n_maps;
  d.n_alloc = n_buf;
  d.out_words_per_map = out_words_per_map;
  d.out_nodes_total = out_nodes_total;
  d.src_words = d_words.p;
  d.src_word_off = d_word_off.p;
  d.src_nodes = d_recs.p;
  d.src_node_off = d_node_off.p;
  d.relocs = d_relocs.p;
  d.src_reloc_off = d_reloc_off.p;
  d.tmpl_graph = d_tmpl_graph.p;
  d.graph_tmpl = d_graph_tmpl.p;
  d.ovr = d_ovr.p;
  d.ovr_off = d_ovr_off.p;
  d.govr = d_govr.p;
  d.govr_off = d_govr_off.p;
  d.new_base = d_new_base.p;
  const size_t ws_mat = fdy_materialize_workspace_bytes(&d);
  CK(d_ws_mat.alloc(ws_mat));
  FD(fdy_materialize(&d, d_out.p, d_dims.p, d_ws_mat.p, ws_mat, d_status.p, stream));
  CK(hipStreamSynchronize(stream));
  CK(hipMemcpy(&status, d_status.p, 4, hipMemcpyDeviceToHost));
  if (status != 0) {
    snprintf(msg, msg_len, "device status %u after derive / materialize", status);
    return 1;
  }
  std::vector<uint32_t> dims((size_t)out_nodes_total * 6);
  CK(hipMemcpy(dims.data(), d_dims.p, dims.size() * 4, hipMemcpyDeviceToHost));

  // 3. one template graph per topology, from the captured words of the template's graph
  std::vector<hipGraph_t> graph(n_templates);
  std::vector<hipGraphExec_t> exec(n_templates);
  std::vector<std::vector<hipGraphNode_t>> nodes(n_templates, std::vector<hipGraphNode_t>(n_nodes));
  std::vector<uint32_t> installs(n_templates, 0);
  for (uint32_t t = 0; t < n_templates; ++t) {
    const uint32_t tg = tmpl_graph[t];
    CK(hipGraphCreate(&graph[t], 0));
    for (uint32_t i = 0; i < n_nodes; ++i) {
      void* params[4];
      hipKernelNodeParams np;
      fill_node_params(&np, params, &captured[(size_t)tg * n_nodes + i], sh.uses_b(sh.bucket(tg), i),
                       sh.grid_x(tg, i), 1, 1, kElems, 1, 1);
      CK(hipGraphAddKernelNode(&nodes[t][i], graph[t], i ? &nodes[t][i - 1] : nullptr, i ? 1 : 0, &np));
    }
    CK(hipGraphInstantiate(&exec[t], graph[t], nullptr, nullptr, 0));
  }

  // what the chain leaves in its last buffer for graph g
  auto simulate = [&](uint32_t g, std::vector<uint64_t>& v) {
    v = init;
    const uint32_t t = sh.bucket(g);
    for (uint32_t i = 0; i < n_nodes; ++i)
      for (uint32_t j = 0; j < kElems; ++j) v[j] = step_value(sh.uses_b(t, i), v[j], sh.k(g, i), j, sh.grid_x(g, i));
  };

  // 4. install and replay every (map, graph) on the executable graph of its template
  std::vector<Args> host_args((size_t)n_graphs * n_nodes);
  std::vector<double> t_install, t_launch, t_copy;
  std::vector<uint64_t> got(kElems), want(kElems);
  uint32_t verified = 0, grid_installs = 0;
  for (uint32_t m = 0; m < n_maps; ++m) {
    double t0 = now_ms();
    CK(hipMemcpy(host_args.data(), d_out.p + (size_t)m * out_words_per_map, out_words_per_map * 8,
                 hipMemcpyDeviceToHost));
    t_copy.push_back(now_ms() - t0);
    for (uint32_t g = 0; g < n_graphs; ++g) {
      Args* a = &host_args[(size_t)g * n_nodes];
      const uint32_t* dm = &dims[(size_t)g * n_nodes * 6];
      const uint32_t t = graph_tmpl[g], tb = sh.bucket(tmpl_graph[t]);
      bool other_grid = false;
      t0 = now_ms();
      for (uint32_t i = 0; i < n_nodes; ++i) {
        void* params[4];
        hipKernelNodeParams np;
        fill_node_params(&np, params, &a[i], sh.uses_b(tb, i), dm[6 * i], dm[6 * i + 1], dm[6 * i + 2],
                         dm[6 * i + 3], dm[6 * i + 4], dm[6 * i + 5]);
        CK(hipGraphExecKernelNodeSetParams(exec[t], nodes[t][i], &np));
        other_grid = other_grid || dm[6 * i] != sh.grid_x(tmpl_graph[t], i);
      }
      t_install.push_back(now_ms() - t0);
      ++installs[t];
      grid_installs += other_grid ? 1 : 0;
      t0 = now_ms();
      CK(hipGraphLaunch(exec[t], stream));
      CK(hipStreamSynchronize(stream));
      t_launch.push_back(now_ms() - t0);
      simulate(g, want);
      CK(hipMemcpy(got.data(), (void*)(uintptr_t)buf_addr(m + 1, n_nodes), kBufBytes, hipMemcpyDeviceToHost));
      if (got != want) {
        snprintf(msg, msg_len, "map %u graph %u (template %u): the last buffer does not hold the chain's result", m,
                 g, t);
        return 1;
      }
      ++verified;
    }
  }
  // set A must be untouched: only its first buffer holds data, the rest the fill pattern
  {
    std::vector<unsigned char> a(slab_bytes);
    CK(hipMemcpy(a.data(), slab[0].p, slab_bytes, hipMemcpyDeviceToHost));
    for (size_t i = kBufBytes; i < slab_bytes; ++i)
      if (a[i] != 0xA5) {
        snprintf(msg, msg_len, "the captured buffer set was written by a replay (byte %zu)", i);
        return 1;
      }
  }

  // 4b. the paper's own form of the in-place update (Section 4.2.1): the target graph's node
  // parameters are set on the template GRAPH and the executable graph is updated from it as a
  // whole (one hipGraphExecUpdate instead of one hipGraphExecKernelNodeSetParams per node).
  // Timed and verified on the first base map for up to eight graphs spread over the topologies.
  std::vector<double> t_update;
  {
    CK(hipMemcpy(host_args.data(), d_out.p, out_words_per_map * 8, hipMemcpyDeviceToHost));
    const uint32_t n_try = 8;
    for (uint32_t q = 0; q < n_try; ++q) {
      const uint32_t g = (uint32_t)((uint64_t)q * (n_graphs - 1) / (n_try - 1));
      Args* a = &host_args[(size_t)g * n_nodes];
      const uint32_t* dm = &dims[(size_t)g * n_nodes * 6];
      const uint32_t t = graph_tmpl[g], tb = sh.bucket(tmpl_graph[t]);
      const double t0 = now_ms();
      for (uint32_t i = 0; i < n_nodes; ++i) {
        void* params[4];
        hipKernelNodeParams np;
        fill_node_params(&np, params, &a[i], sh.uses_b(tb, i), dm[6 * i], dm[6 * i + 1], dm[6 * i + 2],
                         dm[6 * i + 3], dm[6 * i + 4], dm[6 * i + 5]);
        CK(hipGraphKernelNodeSetParams(nodes[t][i], &np));
      }
      hipGraphNode_t err_node = nullptr;
      hipGraphExecUpdateResult res = hipGraphExecUpdateSuccess;
      CK(hipGraphExecUpdate(exec[t], graph[t], &err_node, &res));
      t_update.push_back(now_ms() - t0);
      if (res != hipGraphExecUpdateSuccess) {
        snprintf(msg, msg_len, "hipGraphExecUpdate refused the update (result %d)", (int)res);
        return 1;
      }
      CK(hipGraphLaunch(exec[t], stream));
      CK(hipStreamSynchronize(stream));
      simulate(g, want);
      CK(hipMemcpy(got.data(), (void*)(uintptr_t)buf_addr(1, n_nodes), kBufBytes, hipMemcpyDeviceToHost));
      if (got != want) {
        snprintf(msg, msg_len, "whole-graph update, graph %u: the last buffer does not hold the chain's result", g);
        return 1;
      }
    }
  }

  // 5. the alternative: build and instantiate the graph from scratch
  std::vector<double> t_build;
  for (int rep = 0; rep < 5; ++rep) {
    Args* a = &host_args[0];
    const double t0 = now_ms();
    hipGraph_t g2;
    std::vector<hipGraphNode_t> n2(n_nodes);
    CK(hipGraphCreate(&g2, 0));
    for (uint32_t i = 0; i < n_nodes; ++i) {
      void* params[4];
      hipKernelNodeParams np;
      fill_node_params(&np, params, &a[i], sh.uses_b(sh.bucket(0), i), sh.grid_x(0, i), 1, 1, kElems, 1, 1);
      CK(hipGraphAddKernelNode(&n2[i], g2, i ? &n2[i - 1] : nullptr, i ? 1 : 0, &np));
    }
    hipGraphExec_t e2;
    CK(hipGraphInstantiate(&e2, g2, nullptr, nullptr, 0));
    t_build.push_back(now_ms() - t0);
    CK(hipGraphExecDestroy(e2));
    CK(hipGraphDestroy(g2));
  }
  uint32_t used = 0;
  for (uint32_t t = 0; t < n_templates; ++t) used += installs[t] ? 1 : 0;
  stats[0] = median(t_install);
  stats[1] = *std::min_element(t_install.begin(), t_install.end());
  stats[2] = *std::max_element(t_install.begin(), t_install.end());
  stats[3] = median(t_build);
  stats[4] = median(t_launch);
  stats[5] = verified;
  stats[6] = (double)count;
  stats[7] = median(t_copy);
  stats[8] = median(t_update);
  stats[9] = n_templates;
  stats[10] = used;
  stats[11] = grid_installs;
  for (uint32_t t = 0; t < n_templates; ++t) {
    CK(hipGraphExecDestroy(exec[t]));
    CK(hipGraphDestroy(graph[t]));
  }
  CK(hipStreamDestroy(stream));
  snprintf(msg, msg_len,
           "ok: %u nodes x %u graphs x %u maps, %u topologies each with its own executable graph, launch dimensions "
           "installed; install %.3f ms/graph (min %.3f, max %.3f), whole-graph update %.3f ms/graph, "
           "build+instantiate %.3f ms/graph, launch+sync %.3f ms",
           n_nodes, n_graphs, n_maps, n_templates, stats[0], stats[1], stats[2], stats[8], stats[3], stats[4]);
  return 0;
}
