// arena_graph.hip - the deterministic layout end to end (test program, not part of the library).
//
// Section 4.1.1 / Section 5.1 of the paper: a run that repeats the same sequence of
// allocations inside its reserved range gets the same layout; here the new instance's range
// may start elsewhere (the relaxation this repository targets), and the pointers captured in
// kernel arguments are found and rebased.
//   1. two arenas (fdy_arena.h) at different requested addresses replay one sequence of
//      allocations: offsets inside the arenas must agree, both tables must be valid;
//   2. a hipGraph of chained toy kernels is built on arena A's buffers and instantiated;
//   3. the nodes' argument words are rebased for arena B in one pass (fdy_scan_rebase with
//      A's table and B's bases), installed with hipGraphExecKernelNodeSetParams, replayed:
//      B's buffers hold the chain's results, A's are untouched;
//   4. arena A is reset and the sequence replayed: the same addresses come back;
//   (between 1 and 2) a third arena is given A's recorded table alone (fdy_arena_replay): every
//      allocation lands at the same distance from that arena's base, backed by memory.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "fdy.h"
#include "fdy_arena.h"

namespace {

constexpr uint32_t kN = 777;  // elements per buffer
constexpr int kNodes = 5;

__global__ void arena_kernel(const uint64_t* src, uint64_t* dst, uint32_t k, uint32_t n) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i] * k + i;
}

struct Args {
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
      snprintf(msg, msg_len, "%s failed: %s [%s]", #expr, fdy_strerror(r__),     \
               fdy_arena_last_failure());                                         \
      return 1;                                                                   \
    }                                                                             \
  } while (0)

// the allocation sequence both instances replay: the chain's buffers with odd-sized scratch
// allocations between them
int replay_sequence(fdy_arena* a, std::vector<void*>* bufs) {
  bufs->clear();
  for (int b = 0; b <= kNodes; ++b) {
    void* p = nullptr;
    int rc = fdy_arena_alloc(a, (size_t)kN * 8, 0, &p);
    if (rc != FDY_OK) return rc;
    bufs->push_back(p);
    void* scratch = nullptr;
    rc = fdy_arena_alloc(a, 100 + 37 * (size_t)b, b % 2 ? 4096 : 8, &scratch);
    if (rc != FDY_OK) return rc;
  }
  return FDY_OK;
}

}  // namespace

extern "C" int arena_graph_check(char* msg, int msg_len) {
  hipStream_t stream;
  CK(hipStreamCreate(&stream));
  fdy_arena *A = nullptr, *B = nullptr;
  const uint64_t hint_a = 0x200000000000ull, hint_b = 0x300000000000ull;
  FD(fdy_arena_create(&A, hint_a, 4u << 20));
  FD(fdy_arena_create(&B, hint_b, 4u << 20));
  const uint64_t base_a = fdy_arena_base(A), base_b = fdy_arena_base(B);
  if (base_a == base_b || base_a == 0 || base_b == 0) {
    snprintf(msg, msg_len, "arena bases %llx %llx", (unsigned long long)base_a, (unsigned long long)base_b);
    return 1;
  }
  std::vector<void*> bufs_a, bufs_b;
  FD(replay_sequence(A, &bufs_a));
  FD(replay_sequence(B, &bufs_b));
  const uint32_t n_alloc = fdy_arena_count(A);
  if (n_alloc != 2 * (kNodes + 1) || fdy_arena_count(B) != n_alloc) {
    snprintf(msg, msg_len, "allocation counts differ");
    return 1;
  }
  std::vector<fdy_alloc> ta(n_alloc), tb(n_alloc);
  FD(fdy_arena_table(A, ta.data(), n_alloc));
  FD(fdy_arena_table(B, tb.data(), n_alloc));
  uint32_t bad = 0;
  FD(fdy_table_validate(ta.data(), n_alloc, &bad));
  FD(fdy_table_validate(tb.data(), n_alloc, &bad));
  std::vector<uint64_t> new_base(n_alloc);
  for (uint32_t i = 0; i < n_alloc; ++i) {
    if (ta[i].base - base_a != tb[i].base - base_b || ta[i].size != tb[i].size) {
      snprintf(msg, msg_len, "allocation %u sits at different offsets in the two arenas", i);
      return 1;
    }
    new_base[i] = tb[i].base;
  }
  // capture-window replay from the recording alone: a third arena takes A's table and puts every
  // allocation at the same distance from its own base, without the sequence being issued again
  {
    fdy_arena* R = nullptr;
    FD(fdy_arena_create(&R, 0x280000000000ull, 4u << 20));
    const uint64_t base_r = fdy_arena_base(R);
    std::vector<uint64_t> nb_r(n_alloc);
    std::vector<fdy_alloc> tr(n_alloc);
    FD(fdy_arena_replay(R, ta.data(), n_alloc, base_a, nb_r.data()));
    FD(fdy_arena_table(R, tr.data(), n_alloc));
    for (uint32_t i = 0; i < n_alloc; ++i) {
      if (fdy_arena_count(R) != n_alloc || nb_r[i] != base_r + (ta[i].base - base_a) || tr[i].base != nb_r[i] ||
          tr[i].size != ta[i].size) {
        snprintf(msg, msg_len, "replayed allocation %u is not where the recording puts it", i);
        return 1;
      }
    }
    // the replayed range is backed by memory, the next allocation lands behind it, and the
    // recording cannot be placed a second time over itself
    CK(hipMemset((void*)(uintptr_t)nb_r[n_alloc - 1], 0x5a, (size_t)ta[n_alloc - 1].size));
    void* next = nullptr;
    FD(fdy_arena_alloc(R, 64, 8, &next));
    if ((uint64_t)(uintptr_t)next < nb_r[n_alloc - 1] + ta[n_alloc - 1].size ||
        fdy_arena_replay(R, ta.data(), n_alloc, base_a, nb_r.data()) != FDY_ERR_ORDER ||
        fdy_arena_count(R) != n_alloc + 1) {
      snprintf(msg, msg_len, "the arena's state after a replay is wrong");
      return 1;
    }
    FD(fdy_arena_destroy(R));
  }
  // chain input in both instances, sentinels elsewhere
  std::vector<uint64_t> init(kN), sentinel(kN, 0xA5A5A5A5A5A5A5A5ull);
  for (uint32_t i = 0; i < kN; ++i) init[i] = 11 + 3 * i;
  for (int b = 0; b <= kNodes; ++b) {
    CK(hipMemcpy(bufs_a[b], b == 0 ? init.data() : sentinel.data(), kN * 8, hipMemcpyHostToDevice));
    CK(hipMemcpy(bufs_b[b], b == 0 ? init.data() : sentinel.data(), kN * 8, hipMemcpyHostToDevice));
  }

  // template graph on arena A
  hipGraph_t graph;
  CK(hipGraphCreate(&graph, 0));
  hipGraphNode_t nodes[kNodes];
  Args captured[kNodes];
  for (int i = 0; i < kNodes; ++i) {
    captured[i] = Args{(uint64_t)(uintptr_t)bufs_a[i], (uint64_t)(uintptr_t)bufs_a[i + 1], (uint32_t)(3 + i), kN};
    void* params[4] = {&captured[i].src, &captured[i].dst, &captured[i].k, &captured[i].n};
    hipKernelNodeParams np;
    memset(&np, 0, sizeof np);
    np.func = (void*)arena_kernel;
    np.gridDim = dim3((kN + 255) / 256);
    np.blockDim = dim3(256);
    np.kernelParams = params;
    CK(hipGraphAddKernelNode(&nodes[i], graph, i ? &nodes[i - 1] : nullptr, i ? 1 : 0, &np));
  }
  hipGraphExec_t exec;
  CK(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));

  // rebase the argument words for arena B in one pass; the scratch lives in arena B too
  const uint64_t n_words = kNodes * 3;
  void *d_words = nullptr, *d_table = nullptr, *d_nb = nullptr, *d_out = nullptr, *d_count = nullptr,
       *d_ws = nullptr, *d_status = nullptr;
  const size_t ws_bytes = fdy_scan_workspace_bytes(n_words, n_alloc);
  FD(fdy_arena_alloc(B, n_words * 8, 16, &d_words));
  FD(fdy_arena_alloc(B, n_alloc * sizeof(fdy_alloc), 16, &d_table));
  FD(fdy_arena_alloc(B, n_alloc * 8, 16, &d_nb));
  FD(fdy_arena_alloc(B, n_words * 8, 16, &d_out));
  FD(fdy_arena_alloc(B, 8, 8, &d_count));
  FD(fdy_arena_alloc(B, 4, 8, &d_status));
  FD(fdy_arena_alloc(B, ws_bytes, 256, &d_ws));
  CK(hipMemcpy(d_words, captured, n_words * 8, hipMemcpyHostToDevice));
  CK(hipMemcpy(d_table, ta.data(), n_alloc * sizeof(fdy_alloc), hipMemcpyHostToDevice));
  CK(hipMemcpy(d_nb, new_base.data(), n_alloc * 8, hipMemcpyHostToDevice));
  CK(hipMemset(d_status, 0, 4));
  FD(fdy_scan_rebase((const uint64_t*)d_words, n_words, (const fdy_alloc*)d_table, n_alloc,
                     (const uint64_t*)d_nb, (uint64_t*)d_out, (uint64_t*)d_count, nullptr, d_ws, ws_bytes,
                     (uint32_t*)d_status, stream));
  CK(hipStreamSynchronize(stream));
  uint64_t count = 0;
  uint32_t status = 0;
  Args rebased[kNodes];
  CK(hipMemcpy(&count, d_count, 8, hipMemcpyDeviceToHost));
  CK(hipMemcpy(&status, d_status, 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(rebased, d_out, sizeof rebased, hipMemcpyDeviceToHost));
  if (status != 0 || count != 2 * kNodes) {
    snprintf(msg, msg_len, "%llu pointers rebased (want %d), status %u", (unsigned long long)count, 2 * kNodes,
             status);
    return 1;
  }
  for (int i = 0; i < kNodes; ++i) {
    void* params[4] = {&rebased[i].src, &rebased[i].dst, &rebased[i].k, &rebased[i].n};
    hipKernelNodeParams np;
    memset(&np, 0, sizeof np);
    np.func = (void*)arena_kernel;
    np.gridDim = dim3((kN + 255) / 256);
    np.blockDim = dim3(256);
    np.kernelParams = params;
    CK(hipGraphExecKernelNodeSetParams(exec, nodes[i], &np));
  }
  CK(hipGraphLaunch(exec, stream));
  CK(hipStreamSynchronize(stream));
  std::vector<uint64_t> want(init), got(kN);
  for (int i = 0; i < kNodes; ++i) {
    for (uint32_t j = 0; j < kN; ++j) want[j] = want[j] * (3 + i) + j;
    CK(hipMemcpy(got.data(), bufs_b[i + 1], kN * 8, hipMemcpyDeviceToHost));
    if (got != want) {
      snprintf(msg, msg_len, "arena B buffer %d does not hold the expected values", i + 1);
      return 1;
    }
    CK(hipMemcpy(got.data(), bufs_a[i + 1], kN * 8, hipMemcpyDeviceToHost));
    if (got != sentinel) {
      snprintf(msg, msg_len, "arena A buffer %d was written by the replay", i + 1);
      return 1;
    }
  }
  // capture-window replay: the same sequence after a reset lands on the same addresses
  std::vector<void*> again;
  FD(fdy_arena_reset(A));
  FD(replay_sequence(A, &again));
  if (again != bufs_a) {
    snprintf(msg, msg_len, "the replayed sequence got different addresses");
    return 1;
  }
  // capacity is enforced without side effects
  void* too_big = nullptr;
  if (fdy_arena_alloc(A, fdy_arena_capacity(A), 0, &too_big) != FDY_ERR_CAPACITY ||
      fdy_arena_count(A) != 2 * (kNodes + 1)) {
    snprintf(msg, msg_len, "an allocation beyond the capacity was not refused cleanly");
    return 1;
  }
  CK(hipGraphExecDestroy(exec));
  CK(hipGraphDestroy(graph));
  FD(fdy_arena_destroy(A));
  FD(fdy_arena_destroy(B));
  CK(hipStreamDestroy(stream));
  snprintf(msg, msg_len,
           "ok: arenas at %llx (asked %llx) and %llx (asked %llx), %u allocations at equal offsets, %llu pointers "
           "rebased, graph replayed on the second arena",
           (unsigned long long)base_a, (unsigned long long)hint_a, (unsigned long long)base_b,
           (unsigned long long)hint_b, n_alloc, (unsigned long long)count);
  return 0;
}
