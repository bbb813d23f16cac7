// install_scale.hip - hipGraph install at the scale of a decode graph (test program, not part
// of the library).
//
// Section 4.2.1 / Section 5.3 and Table 2 of the paper: a target graph is brought up by
// applying its node parameters to the template's executable graph (in-place update), which
// the paper times per graph against building and instantiating the graph from scratch.
// This program does the same with arguments produced by libfdy, at the node count of one
// dense-decode graph:
//   1. a template hipGraph of `n_nodes` chained toy kernels is built on buffer set A (one
//      slab, node i reads buffer i and writes buffer i + 1) and instantiated once;
//   2. the nodes' argument buffers (24 bytes each) are scanned against set A's allocation
//      table, fingerprinted (every graph shares the one topology) and materialized for
//      `n_maps` other slabs and `n_graphs` graphs that differ in two 32-bit scalars each;
//   3. for every (map, graph) the materialized words are copied to the host once per map and
//      installed node by node with hipGraphExecKernelNodeSetParams; the install is timed on
//      the host clock; the executable graph is launched and the last buffer of the map's slab
//      is compared with a host simulation of the chain; set A must stay untouched;
//   4. for comparison, building and instantiating a fresh graph of the same nodes is timed.
// Results go to `stats`: [0] install ms per graph (median), [1] min, [2] max, [3] build +
// instantiate ms per graph (median of 5), [4] launch + sync ms per graph (median), [5] number of
// (map, graph) pairs verified, [6] relocations per graph, [7] device-to-host copy ms per map,
// [8] ms per graph of the whole-graph form of the update (set the parameters on the graph's nodes,
// then one hipGraphExecUpdate; median over up to eight graphs).  `stats` holds 9 doubles.
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

__global__ void chain_kernel(const uint64_t* src, uint64_t* dst, uint32_t k, uint32_t n) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i] * k + i;
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

uint32_t default_k(uint32_t node) { return 2 + node % 5; }
// the two nodes whose scalar graph g overrides, and the value
uint32_t ovr_node(uint32_t g, int which, uint32_t n_nodes) { return (which ? 7 * g + 3 : g) % n_nodes; }
uint32_t ovr_value(uint32_t g, int which) { return 100 + 2 * g + which; }

void fill_node_params(hipKernelNodeParams* np, void** params, Args* a) {
  params[0] = &a->src;
  params[1] = &a->dst;
  params[2] = &a->k;
  params[3] = &a->n;
  memset(np, 0, sizeof *np);
  np->func = (void*)chain_kernel;
  np->gridDim = dim3(1);
  np->blockDim = dim3(kElems);
  np->kernelParams = params;
}

}  // namespace

extern "C" int install_scale_check(uint32_t n_nodes, uint32_t n_graphs, uint32_t n_maps, double* stats,
                                   char* msg, int msg_len) {
  if (n_nodes < 1 || n_nodes > 4096 || n_graphs < 1 || n_graphs > 512 || n_maps < 1 || n_maps > 8) {
    snprintf(msg, msg_len, "sizes out of range");
    return 1;
  }
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

  // 1. template graph on set A
  std::vector<Args> captured(n_nodes);
  std::vector<hipGraphNode_t> nodes(n_nodes);
  hipGraph_t graph;
  CK(hipGraphCreate(&graph, 0));
  for (uint32_t i = 0; i < n_nodes; ++i) {
    captured[i] = Args{buf_addr(0, i), buf_addr(0, i + 1), default_k(i), kElems};
    void* params[4];
    hipKernelNodeParams np;
    fill_node_params(&np, params, &captured[i]);
    CK(hipGraphAddKernelNode(&nodes[i], graph, i ? &nodes[i - 1] : nullptr, i ? 1 : 0, &np));
  }
  hipGraphExec_t exec;
  CK(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));

  // 2. scan, fingerprint, materialize
  std::vector<fdy_alloc> table(n_buf);
  for (uint32_t b = 0; b < n_buf; ++b) table[b] = fdy_alloc{buf_addr(0, b), kBufBytes};
  uint32_t bad = 0;
  FD(fdy_table_validate(table.data(), n_buf, &bad));
  std::vector<uint64_t> new_base((size_t)n_maps * n_buf);
  for (uint32_t m = 0; m < n_maps; ++m)
    for (uint32_t b = 0; b < n_buf; ++b) new_base[(size_t)m * n_buf + b] = buf_addr(m + 1, b);
  const uint64_t n_words = (uint64_t)n_nodes * 3;
  std::vector<fdy_node> recs(n_nodes);
  for (uint32_t i = 0; i < n_nodes; ++i) {
    memset(&recs[i], 0, sizeof recs[i]);
    recs[i].kernel_id = 0x1000 + i % 16;  // sixteen kernels per layer
    recs[i].grid[0] = recs[i].grid[1] = recs[i].grid[2] = 1;
    recs[i].block[0] = kElems;
    recs[i].block[1] = recs[i].block[2] = 1;
    recs[i].blob_len = sizeof(Args);
  }
  // n_graphs captured graphs with identical node records: one template
  std::vector<fdy_node> all_recs;
  std::vector<uint64_t> node_off(n_graphs + 1), ovr_off(n_graphs + 1), zeros(n_graphs + 1, 0);
  std::vector<fdy_ovr32> ovr;
  for (uint32_t g = 0; g < n_graphs; ++g) {
    node_off[g] = all_recs.size();
    all_recs.insert(all_recs.end(), recs.begin(), recs.end());
    ovr_off[g] = ovr.size();
    // ascending by byte offset; when both scalars fall on one node the second wins, as in the
    // host simulation below
    const uint32_t n0 = ovr_node(g, 0, n_nodes), n1 = ovr_node(g, 1, n_nodes);
    if (n0 < n1) ovr.push_back(fdy_ovr32{n0 * 24 + 16, ovr_value(g, 0)});
    ovr.push_back(fdy_ovr32{n1 * 24 + 16, ovr_value(g, 1)});
    if (n0 > n1) ovr.push_back(fdy_ovr32{n0 * 24 + 16, ovr_value(g, 0)});
  }
  node_off[n_graphs] = all_recs.size();
  ovr_off[n_graphs] = ovr.size();

  DevBuf<uint64_t> d_words, d_count, d_word_off, d_reloc_off, d_new_base, d_out, d_ovr_off, d_zero_off, d_node_off,
      d_keys;
  DevBuf<fdy_alloc> d_table;
  DevBuf<fdy_reloc> d_relocs;
  DevBuf<fdy_node> d_recs;
  DevBuf<uint32_t> d_status, d_tmpl_graph, d_graph_tmpl, d_n_tmpl;
  DevBuf<fdy_ovr32> d_ovr;
  DevBuf<unsigned char> d_ws_scan, d_ws_mat;
  CK(d_words.alloc(n_words + 2));
  CK(hipMemcpy(d_words.p, captured.data(), n_words * 8, hipMemcpyHostToDevice));
  CK(d_table.upload(table));
  CK(d_relocs.alloc(n_words));
  CK(d_count.alloc(1));
  CK(d_status.alloc(1));
  CK(hipMemset(d_status.p, 0, 4));
  const size_t ws_scan = fdy_scan_workspace_bytes(n_words, n_buf);
  CK(d_ws_scan.alloc(ws_scan));
  FD(fdy_scan_pointers(d_words.p, n_words, d_table.p, n_buf, d_relocs.p, n_words, d_count.p, nullptr,
                       d_ws_scan.p, ws_scan, d_status.p, stream));
  const std::vector<uint64_t> word_off = {0, n_words};
  CK(d_word_off.upload(word_off));
  CK(d_reloc_off.alloc(2));
  FD(fdy_reloc_segment(d_relocs.p, d_count.p, n_words, d_word_off.p, 2, d_reloc_off.p, stream));
  CK(d_recs.upload(all_recs));
  CK(d_node_off.upload(node_off));
  CK(d_keys.alloc(n_graphs));
  CK(d_graph_tmpl.alloc(n_graphs));
  CK(d_tmpl_graph.alloc(n_graphs));
  CK(d_n_tmpl.alloc(1));
  FD(fdy_fingerprint(d_recs.p, d_node_off.p, n_graphs, FDY_FP_ALL, d_keys.p, d_graph_tmpl.p, d_tmpl_graph.p,
                     d_n_tmpl.p, nullptr, 0, stream));
  CK(hipStreamSynchronize(stream));
  uint32_t n_templates = 0, status = 0;
  uint64_t count = 0;
  CK(hipMemcpy(&n_templates, d_n_tmpl.p, 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(&count, d_count.p, 8, hipMemcpyDeviceToHost));
  if (n_templates != 1 || count != 2ull * n_nodes) {
    snprintf(msg, msg_len, "%u templates (want 1), %llu pointers (want %u)", n_templates,
             (unsigned long long)count, 2 * n_nodes);
    return 1;
  }
  // every captured graph has the same words here, so the archive holds the template's once:
  // source graph 0 = the template; tmpl_graph from the fingerprint names graph 0
  CK(d_ovr.upload(ovr));
  CK(d_ovr_off.upload(ovr_off));
  CK(d_zero_off.upload(zeros));
  CK(d_new_base.upload(new_base));
  const uint64_t out_words_per_map = n_words * n_graphs;
  CK(d_out.alloc((size_t)out_words_per_map * n_maps + 2));
  fdy_mat_desc d;
  memset(&d, 0, sizeof d);
  d.n_src_graphs = 1;
  d.n_templates = 1;
  d.n_graphs = n_graphs;
  d.n_maps = n_maps;
  d.n_alloc = n_buf;
  d.out_words_per_map = out_words_per_map;
  d.src_words = d_words.p;
  d.src_word_off = d_word_off.p;
  d.src_node_off = d_zero_off.p;
  d.relocs = d_relocs.p;
  d.src_reloc_off = d_reloc_off.p;
  d.tmpl_graph = d_tmpl_graph.p;
  d.graph_tmpl = d_graph_tmpl.p;
  d.ovr = d_ovr.p;
  d.ovr_off = d_ovr_off.p;
  d.govr_off = d_zero_off.p;
  d.new_base = d_new_base.p;
  const size_t ws_mat = fdy_materialize_workspace_bytes(&d);
  CK(d_ws_mat.alloc(ws_mat));
  FD(fdy_materialize(&d, d_out.p, nullptr, d_ws_mat.p, ws_mat, d_status.p, stream));
  CK(hipStreamSynchronize(stream));
  CK(hipMemcpy(&status, d_status.p, 4, hipMemcpyDeviceToHost));
  if (status != 0) {
    snprintf(msg, msg_len, "materialize status %u", status);
    return 1;
  }

  // 3. install and replay every (map, graph)
  std::vector<Args> host_args((size_t)n_graphs * n_nodes);
  std::vector<double> t_install, t_launch, t_copy;
  std::vector<uint64_t> got(kElems), want(kElems);
  uint32_t verified = 0;
  for (uint32_t m = 0; m < n_maps; ++m) {
    double t0 = now_ms();
    CK(hipMemcpy(host_args.data(), d_out.p + (size_t)m * out_words_per_map, out_words_per_map * 8,
                 hipMemcpyDeviceToHost));
    t_copy.push_back(now_ms() - t0);
    for (uint32_t g = 0; g < n_graphs; ++g) {
      Args* a = &host_args[(size_t)g * n_nodes];
      t0 = now_ms();
      for (uint32_t i = 0; i < n_nodes; ++i) {
        void* params[4];
        hipKernelNodeParams np;
        fill_node_params(&np, params, &a[i]);
        CK(hipGraphExecKernelNodeSetParams(exec, nodes[i], &np));
      }
      t_install.push_back(now_ms() - t0);
      t0 = now_ms();
      CK(hipGraphLaunch(exec, stream));
      CK(hipStreamSynchronize(stream));
      t_launch.push_back(now_ms() - t0);
      // host simulation of the chain with this graph's scalars
      want = init;
      for (uint32_t i = 0; i < n_nodes; ++i) {
        uint32_t k = default_k(i);
        if (i == ovr_node(g, 0, n_nodes)) k = ovr_value(g, 0);
        if (i == ovr_node(g, 1, n_nodes)) k = ovr_value(g, 1);
        for (uint32_t j = 0; j < kElems; ++j) want[j] = want[j] * k + j;
      }
      CK(hipMemcpy(got.data(), (void*)(uintptr_t)buf_addr(m + 1, n_nodes), kBufBytes, hipMemcpyDeviceToHost));
      if (got != want) {
        snprintf(msg, msg_len, "map %u graph %u: the last buffer does not hold the chain's result", m, g);
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

  // 3b. the paper's own form of the in-place update (Section 4.2.1): the target graph's node
  // parameters are set on the template GRAPH and the executable graph is updated from it as a
  // whole (one hipGraphExecUpdate instead of one hipGraphExecKernelNodeSetParams per node).
  // Timed and verified on the first base map for up to eight graphs.
  std::vector<double> t_update;
  {
    CK(hipMemcpy(host_args.data(), d_out.p, out_words_per_map * 8, hipMemcpyDeviceToHost));
    const uint32_t n_try = n_graphs < 8 ? n_graphs : 8;
    for (uint32_t g = 0; g < n_try; ++g) {
      Args* a = &host_args[(size_t)g * n_nodes];
      const double t0 = now_ms();
      for (uint32_t i = 0; i < n_nodes; ++i) {
        void* params[4];
        hipKernelNodeParams np;
        fill_node_params(&np, params, &a[i]);
        CK(hipGraphKernelNodeSetParams(nodes[i], &np));
      }
      hipGraphNode_t err_node = nullptr;
      hipGraphExecUpdateResult res = hipGraphExecUpdateSuccess;
      CK(hipGraphExecUpdate(exec, graph, &err_node, &res));
      t_update.push_back(now_ms() - t0);
      if (res != hipGraphExecUpdateSuccess) {
        snprintf(msg, msg_len, "hipGraphExecUpdate refused the update (result %d)", (int)res);
        return 1;
      }
      CK(hipGraphLaunch(exec, stream));
      CK(hipStreamSynchronize(stream));
      want = init;
      for (uint32_t i = 0; i < n_nodes; ++i) {
        uint32_t k = default_k(i);
        if (i == ovr_node(g, 0, n_nodes)) k = ovr_value(g, 0);
        if (i == ovr_node(g, 1, n_nodes)) k = ovr_value(g, 1);
        for (uint32_t j = 0; j < kElems; ++j) want[j] = want[j] * k + j;
      }
      CK(hipMemcpy(got.data(), (void*)(uintptr_t)buf_addr(1, n_nodes), kBufBytes, hipMemcpyDeviceToHost));
      if (got != want) {
        snprintf(msg, msg_len, "whole-graph update, graph %u: the last buffer does not hold the chain's result", g);
        return 1;
      }
    }
  }

  // 4. the alternative: build and instantiate the graph from scratch
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
      fill_node_params(&np, params, &a[i]);
      CK(hipGraphAddKernelNode(&n2[i], g2, i ? &n2[i - 1] : nullptr, i ? 1 : 0, &np));
    }
    hipGraphExec_t e2;
    CK(hipGraphInstantiate(&e2, g2, nullptr, nullptr, 0));
    t_build.push_back(now_ms() - t0);
    CK(hipGraphExecDestroy(e2));
    CK(hipGraphDestroy(g2));
  }
  stats[0] = median(t_install);
  stats[1] = *std::min_element(t_install.begin(), t_install.end());
  stats[2] = *std::max_element(t_install.begin(), t_install.end());
  stats[3] = median(t_build);
  stats[4] = median(t_launch);
  stats[5] = verified;
  stats[6] = (double)count;
  stats[7] = median(t_copy);
  stats[8] = median(t_update);
  CK(hipGraphExecDestroy(exec));
  CK(hipGraphDestroy(graph));
  CK(hipStreamDestroy(stream));
  snprintf(msg, msg_len,
           "ok: %u nodes x %u graphs x %u maps installed and replayed; install %.3f ms/graph (min %.3f, max %.3f), "
           "whole-graph update %.3f ms/graph, build+instantiate %.3f ms/graph, launch+sync %.3f ms",
           n_nodes, n_graphs, n_maps, stats[0], stats[1], stats[2], stats[8], stats[3], stats[4]);
  return 0;
}
