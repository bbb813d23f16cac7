// toy_graph.hip - tiny end-to-end check (test program, not part of the library).
//
// Section 4.2.1 / Section 5.3 of the paper: at replay the target graph's node parameters are
// applied to the template's executable graph without re-instantiation.  This program does
// that with arguments produced by libfdy:
//   1. a hipGraph of three chained toy kernels is built explicitly on buffer set A and
//      instantiated once (the "template");
//   2. the kernels' argument buffers (24 bytes each: src pointer, dst pointer, k, n) are
//      scanned against the allocation table of set A (fdy_scan_pointers), segmented
//      (fdy_reloc_segment) and materialized (fdy_materialize) for buffer set B, with one
//      32-bit override (k of the middle node);
//   3. the materialized words are installed with hipGraphExecKernelNodeSetParams and the
//      executable graph is launched;
//   4. set B must hold the chain's results (with the overridden k), set A must be untouched.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "fdy.h"

namespace {

constexpr uint32_t kN = 1000;    // elements per buffer
constexpr int kNodes = 3;

__global__ void toy_kernel(const uint64_t* src, uint64_t* dst, uint32_t k, uint32_t n) {
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
};

}  // namespace

extern "C" int toy_graph_check(char* msg, int msg_len) {
  hipStream_t stream;
  CK(hipStreamCreate(&stream));
  // buffer sets: node i reads buf[i], writes buf[i+1]
  DevBuf<uint64_t> A[kNodes + 1], B[kNodes + 1];
  std::vector<uint64_t> init(kN), sentinel(kN, 0xA5A5A5A5A5A5A5A5ull);
  for (uint32_t i = 0; i < kN; ++i) init[i] = 3 + i;
  for (int b = 0; b <= kNodes; ++b) {
    CK(A[b].alloc(kN));
    CK(B[b].alloc(kN));
    CK(hipMemcpy(A[b].p, b == 0 ? init.data() : sentinel.data(), kN * 8, hipMemcpyHostToDevice));
    CK(hipMemcpy(B[b].p, b == 0 ? init.data() : sentinel.data(), kN * 8, hipMemcpyHostToDevice));
  }
  const uint32_t ks[kNodes] = {2, 5, 7};
  const uint32_t k_override = 11;  // for the middle node of the materialized graph

  // 1. template graph on set A
  hipGraph_t graph;
  CK(hipGraphCreate(&graph, 0));
  hipGraphNode_t nodes[kNodes];
  Args captured[kNodes];
  for (int i = 0; i < kNodes; ++i) {
    captured[i] = Args{(uint64_t)(uintptr_t)A[i].p, (uint64_t)(uintptr_t)A[i + 1].p, ks[i], kN};
    void* params[4] = {&captured[i].src, &captured[i].dst, &captured[i].k, &captured[i].n};
    hipKernelNodeParams np;
    memset(&np, 0, sizeof np);
    np.func = (void*)toy_kernel;
    np.gridDim = dim3((kN + 255) / 256);
    np.blockDim = dim3(256);
    np.kernelParams = params;
    CK(hipGraphAddKernelNode(&nodes[i], graph, i ? &nodes[i - 1] : nullptr, i ? 1 : 0, &np));
  }
  hipGraphExec_t exec;
  CK(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));

  // 2. scan + materialize the argument words for set B
  std::vector<fdy_alloc> table;
  std::vector<uint64_t> new_base_by_addr;
  {
    std::vector<std::pair<uint64_t, uint64_t>> ab;  // (A address, B address)
    for (int b = 0; b <= kNodes; ++b) ab.push_back({(uint64_t)(uintptr_t)A[b].p, (uint64_t)(uintptr_t)B[b].p});
    std::sort(ab.begin(), ab.end());
    for (auto& x : ab) {
      table.push_back(fdy_alloc{x.first, (uint64_t)kN * 8});
      new_base_by_addr.push_back(x.second);
    }
  }
  uint32_t bad = 0;
  FD(fdy_table_validate(table.data(), (uint32_t)table.size(), &bad));
  const uint32_t n_words = kNodes * 3, n_alloc = (uint32_t)table.size();
  DevBuf<uint64_t> d_words, d_count, d_word_off, d_reloc_off, d_new_base, d_out, d_ovr_off, d_zero_off;
  DevBuf<fdy_alloc> d_table;
  DevBuf<fdy_reloc> d_relocs;
  DevBuf<uint32_t> d_status, d_tmpl_graph, d_graph_tmpl;
  DevBuf<fdy_ovr32> d_ovr;
  DevBuf<unsigned char> d_ws_scan, d_ws_mat;
  CK(d_words.alloc(n_words + 1));
  CK(d_table.alloc(n_alloc));
  CK(d_relocs.alloc(n_words));
  CK(d_count.alloc(1));
  CK(d_status.alloc(1));
  CK(hipMemcpy(d_words.p, captured, sizeof captured, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_table.p, table.data(), table.size() * sizeof(fdy_alloc), hipMemcpyHostToDevice));
  CK(hipMemset(d_status.p, 0, 4));
  const size_t ws_scan = fdy_scan_workspace_bytes(n_words, n_alloc);
  CK(d_ws_scan.alloc(ws_scan));
  FD(fdy_scan_pointers(d_words.p, n_words, d_table.p, n_alloc, d_relocs.p, n_words, d_count.p,
                       nullptr, d_ws_scan.p, ws_scan, d_status.p, stream));
  const uint64_t word_off[2] = {0, n_words}, zeros[2] = {0, 0}, ovr_off[2] = {0, 1};
  CK(d_word_off.alloc(2));
  CK(d_reloc_off.alloc(2));
  CK(d_zero_off.alloc(2));
  CK(d_ovr_off.alloc(2));
  CK(hipMemcpy(d_word_off.p, word_off, 16, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_zero_off.p, zeros, 16, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_ovr_off.p, ovr_off, 16, hipMemcpyHostToDevice));
  FD(fdy_reloc_segment(d_relocs.p, d_count.p, n_words, d_word_off.p, 2, d_reloc_off.p, stream));
  const fdy_ovr32 ovr = {1 * 24 + 16, k_override};  // field k of node 1
  const uint32_t zero32 = 0;
  CK(d_ovr.alloc(1));
  CK(d_tmpl_graph.alloc(1));
  CK(d_graph_tmpl.alloc(1));
  CK(d_new_base.alloc(n_alloc));
  CK(d_out.alloc(n_words + 1));
  CK(hipMemcpy(d_ovr.p, &ovr, sizeof ovr, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_tmpl_graph.p, &zero32, 4, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_graph_tmpl.p, &zero32, 4, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_new_base.p, new_base_by_addr.data(), n_alloc * 8, hipMemcpyHostToDevice));
  fdy_mat_desc d;
  memset(&d, 0, sizeof d);
  d.n_src_graphs = 1;
  d.n_templates = 1;
  d.n_graphs = 1;
  d.n_maps = 1;
  d.n_alloc = n_alloc;
  d.out_words_per_map = n_words;
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
  uint64_t count = 0;
  uint32_t status = 0;
  Args materialized[kNodes];
  CK(hipMemcpy(&count, d_count.p, 8, hipMemcpyDeviceToHost));
  CK(hipMemcpy(&status, d_status.p, 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(materialized, d_out.p, sizeof materialized, hipMemcpyDeviceToHost));
  if (status != 0 || count != 2 * kNodes) {
    snprintf(msg, msg_len, "scan found %llu pointers (want %d), status %u", (unsigned long long)count,
             2 * kNodes, status);
    return 1;
  }

  // 3. install into the executable template graph, replay
  for (int i = 0; i < kNodes; ++i) {
    void* params[4] = {&materialized[i].src, &materialized[i].dst, &materialized[i].k, &materialized[i].n};
    hipKernelNodeParams np;
    memset(&np, 0, sizeof np);
    np.func = (void*)toy_kernel;
    np.gridDim = dim3((kN + 255) / 256);
    np.blockDim = dim3(256);
    np.kernelParams = params;
    CK(hipGraphExecKernelNodeSetParams(exec, nodes[i], &np));
  }
  CK(hipGraphLaunch(exec, stream));
  CK(hipStreamSynchronize(stream));

  // 4. check: set B holds the chain with the overridden k, set A is untouched
  std::vector<uint64_t> want(init), got(kN);
  for (int i = 0; i < kNodes; ++i) {
    const uint32_t k = i == 1 ? k_override : ks[i];
    for (uint32_t j = 0; j < kN; ++j) want[j] = want[j] * k + j;
    CK(hipMemcpy(got.data(), B[i + 1].p, kN * 8, hipMemcpyDeviceToHost));
    if (got != want) {
      snprintf(msg, msg_len, "buffer B[%d] does not hold the expected values", i + 1);
      return 1;
    }
    CK(hipMemcpy(got.data(), A[i + 1].p, kN * 8, hipMemcpyDeviceToHost));
    if (got != sentinel) {
      snprintf(msg, msg_len, "buffer A[%d] was written by the replay", i + 1);
      return 1;
    }
  }
  CK(hipGraphExecDestroy(exec));
  CK(hipGraphDestroy(graph));
  CK(hipStreamDestroy(stream));
  snprintf(msg, msg_len, "ok: %d nodes, %llu pointers rebased, 1 override, replayed on the second buffer set",
           kNodes, (unsigned long long)count);
  return 0;
}
