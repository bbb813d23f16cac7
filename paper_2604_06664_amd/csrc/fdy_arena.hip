// fdy_arena.hip - deterministic bump allocator over HIP virtual memory management.
//
// Section 4.1.1 / Section 5.1: one reserved address range, allocations placed one after
// another, the record of them is the allocation table.  Physical memory is mapped behind
// the whole range at creation (one handle, one map call), so placing an allocation is
// arithmetic on the host and never touches the driver.
#include <hip/hip_runtime.h>

#include <stdio.h>

#include <new>
#include <vector>

#include "fdy_arena.h"

struct fdy_arena {
  void* base = nullptr;
  size_t capacity = 0;  // reserved = mapped bytes
  size_t used = 0;      // bump pointer (bytes from base)
  hipMemGenericAllocationHandle_t handle{};
  bool have_handle = false, mapped = false;
  std::vector<fdy_alloc> table;
};

namespace {

// the driver call that failed last, with the driver's own text (diagnostics only)
thread_local char g_failure[160] = "";

bool failed(hipError_t e, const char* what) {
  if (e == hipSuccess) return false;
  snprintf(g_failure, sizeof g_failure, "%s: %s", what, hipGetErrorString(e));
  (void)hipGetLastError();
  return true;
}

int release(fdy_arena* a) {
  int rc = FDY_OK;
  if (a->mapped && hipMemUnmap(a->base, a->capacity) != hipSuccess) rc = FDY_ERR_HIP;
  if (a->have_handle && hipMemRelease(a->handle) != hipSuccess) rc = FDY_ERR_HIP;
  if (a->base && hipMemAddressFree(a->base, a->capacity) != hipSuccess) rc = FDY_ERR_HIP;
  delete a;
  return rc;
}

}  // namespace

namespace {

// One attempt at `va_hint` (0: anywhere).  On failure nothing stays reserved.
int create_at(fdy_arena** out, uint64_t va_hint, size_t cap, size_t gran, const hipMemAllocationProp& prop,
              int dev) {
  fdy_arena* a = new (std::nothrow) fdy_arena;
  if (!a) return FDY_ERR_HIP;
  a->capacity = cap;
  if (failed(hipMemAddressReserve(&a->base, cap, gran, (void*)(uintptr_t)va_hint, 0), "hipMemAddressReserve")) {
    a->base = nullptr;
    release(a);
    return FDY_ERR_HIP;
  }
  if (failed(hipMemCreate(&a->handle, cap, &prop, 0), "hipMemCreate")) {
    release(a);
    return FDY_ERR_HIP;
  }
  a->have_handle = true;
  if (failed(hipMemMap(a->base, cap, 0, a->handle, 0), "hipMemMap")) {
    release(a);
    return FDY_ERR_HIP;
  }
  a->mapped = true;
  hipMemAccessDesc acc{};
  acc.location.type = hipMemLocationTypeDevice;
  acc.location.id = dev;
  acc.flags = hipMemAccessFlagsProtReadWrite;
  if (failed(hipMemSetAccess(a->base, cap, &acc, 1), "hipMemSetAccess")) {
    release(a);
    return FDY_ERR_HIP;
  }
  *out = a;
  return FDY_OK;
}

}  // namespace

extern "C" int fdy_arena_create(fdy_arena** out, uint64_t va_hint, size_t capacity_bytes) {
  if (!out || capacity_bytes == 0) return FDY_ERR_INVALID_ARG;
  *out = nullptr;
  g_failure[0] = 0;
  (void)hipGetLastError();
  int dev = 0;
  if (failed(hipGetDevice(&dev), "hipGetDevice")) return FDY_ERR_HIP;
  hipMemAllocationProp prop{};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = dev;
  size_t gran = 0;
  if (failed(hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityRecommended),
             "hipMemGetAllocationGranularity") ||
      gran == 0)
    return FDY_ERR_HIP;
  const size_t cap = (capacity_bytes + gran - 1) / gran * gran;
  // The requested address is a wish.  A driver may refuse it outright, or grant the
  // reservation and then refuse access to it (measured on MI355X: addresses outside
  // 0x1000_0000_0000 .. 0x4fff_ffff_ffff reserve and map, but cannot be made accessible);
  // either way the arena is then placed wherever the driver likes.
  int rc = create_at(out, va_hint, cap, gran, prop, dev);
  if (rc != FDY_OK && va_hint != 0) rc = create_at(out, 0, cap, gran, prop, dev);
  return rc;
}

extern "C" const char* fdy_arena_last_failure(void) { return g_failure; }

extern "C" uint64_t fdy_arena_base(const fdy_arena* a) { return a ? (uint64_t)(uintptr_t)a->base : 0; }
extern "C" size_t fdy_arena_capacity(const fdy_arena* a) { return a ? a->capacity : 0; }

extern "C" int fdy_arena_alloc(fdy_arena* a, size_t bytes, size_t alignment, void** d_ptr) {
  if (!a || !d_ptr || bytes == 0) return FDY_ERR_INVALID_ARG;
  if (alignment == 0) alignment = 512;
  if (alignment < 8 || (alignment & (alignment - 1))) return FDY_ERR_INVALID_ARG;
  const size_t at = (a->used + alignment - 1) & ~(alignment - 1);
  if (at < a->used || at > a->capacity || bytes > a->capacity - at) return FDY_ERR_CAPACITY;
  if (a->table.size() >= 0xffffffffu) return FDY_ERR_CAPACITY;
  a->used = at + bytes;
  const uint64_t base = (uint64_t)(uintptr_t)a->base + at;
  a->table.push_back(fdy_alloc{base, (uint64_t)bytes});
  *d_ptr = (void*)(uintptr_t)base;
  return FDY_OK;
}

extern "C" uint32_t fdy_arena_count(const fdy_arena* a) { return a ? (uint32_t)a->table.size() : 0; }

extern "C" int fdy_arena_table(const fdy_arena* a, fdy_alloc* h_table, uint32_t capacity) {
  if (!a || (capacity && !h_table)) return FDY_ERR_INVALID_ARG;
  const size_t n = a->table.size() < capacity ? a->table.size() : capacity;
  for (size_t i = 0; i < n; ++i) h_table[i] = a->table[i];
  return FDY_OK;
}

extern "C" int fdy_arena_reset(fdy_arena* a) {
  if (!a) return FDY_ERR_INVALID_ARG;
  a->used = 0;
  a->table.clear();
  return FDY_OK;
}

extern "C" int fdy_arena_replay(fdy_arena* a, const fdy_alloc* h_recorded, uint32_t n, uint64_t recorded_base,
                                uint64_t* h_new_base) {
  if (!a) return FDY_ERR_INVALID_ARG;
  if (n == 0) return FDY_OK;
  if (a->table.size() + (size_t)n > 0xffffffffu) return FDY_ERR_CAPACITY;
  const uint64_t base = (uint64_t)(uintptr_t)a->base;
  const int rc = fdy_layout_replay(h_recorded, n, recorded_base, base, a->capacity, a->used, h_new_base);
  if (rc != FDY_OK) return rc;
  for (uint32_t i = 0; i < n; ++i) a->table.push_back(fdy_alloc{h_new_base[i], h_recorded[i].size});
  a->used = (size_t)(h_new_base[n - 1] + h_recorded[n - 1].size - base);
  return FDY_OK;
}

extern "C" int fdy_arena_destroy(fdy_arena* a) {
  if (!a) return FDY_OK;
  (void)hipGetLastError();
  return release(a);
}
