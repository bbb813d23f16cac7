// fdy_api.hip - version, error strings, host-side table validation and layout inversion,
// tuning knobs.
#include <algorithm>
#include <vector>

#include "fdy_device.hpp"
#include "fdy_internal.h"

namespace {
int g_tune[FDY_TUNE_COUNT] = {
    /* SCAN_TOP_LOG2   */ 14,
    /* SCAN_WG_PER_CU  */ 1,
    /* SCAN_SPIN_LIMIT */ 1 << 20,
    /* MAT_MAP_GROUP     */ 0,
    /* SCAN_SMALL_LOG2 */ 12,
    /* MAT_SELF_WGS    */ 1024,
    /* MAT_ONCE_TILES  */ 4096,
    0};
const int g_tune_lo[FDY_TUNE_COUNT] = {1, 1, 0, 0, 0, 0, 1, 0};
const int g_tune_hi[FDY_TUNE_COUNT] = {14, 16, 1 << 30, 64, 31, 1 << 30, 1 << 30, 0};
}  // namespace

extern "C" int fdy__tune_get(int knob) {
  return knob >= 0 && knob < FDY_TUNE_COUNT ? g_tune[knob] : -1;
}

extern "C" int fdy__tune_set(int knob, int value) {
  if (knob < 0 || knob >= FDY_TUNE_COUNT) return -1;
  if (value < g_tune_lo[knob] || value > g_tune_hi[knob]) return -1;
  const int old = g_tune[knob];
  g_tune[knob] = value;
  return old;
}

extern "C" int fdy_version(void) { return FDY_VERSION; }

extern "C" const char* fdy_strerror(int code) {
  switch (code) {
    case FDY_OK: return "ok";
    case FDY_ERR_INVALID_ARG: return "invalid argument (null or misaligned pointer, size out of range)";
    case FDY_ERR_TABLE: return "allocation table is not strictly ascending, non-empty, non-wrapping and non-overlapping";
    case FDY_ERR_CAPACITY: return "relocation capacity exceeded";
    case FDY_ERR_HIP: return "a HIP call or kernel launch failed";
    case FDY_ERR_WORKSPACE: return "workspace is null, misaligned or too small";
    case FDY_ERR_ORDER: return "a list is not strictly ascending by location";
    case FDY_ERR_IO: return "a file could not be opened, mapped or written";
    case FDY_ERR_FORMAT: return "not an archive, or a damaged container";
    case FDY_ERR_CHECKSUM: return "a stored sum does not match the bytes";
    case FDY_ERR_CONTENT: return "the sections of the archive contradict each other";
    default: return "unknown fdy error code";
  }
}

extern "C" int fdy_table_validate(const fdy_alloc* h_table, uint32_t n_alloc, uint32_t* h_bad_index) {
  if (n_alloc == 0) return FDY_OK;
  if (!h_table) return FDY_ERR_INVALID_ARG;
  uint64_t prev_end = 0;
  for (uint32_t i = 0; i < n_alloc; ++i) {
    const uint64_t b = h_table[i].base, s = h_table[i].size;
    const uint64_t end = b + s;
    // size >= 1 and no wrap  <=>  end > b ; sorted + disjoint  <=>  b >= previous end
    // (and strictly above the previous base, which previous size >= 1 already implies)
    if (!(end > b) || (i > 0 && b < prev_end)) {
      if (h_bad_index) *h_bad_index = i;
      return FDY_ERR_TABLE;
    }
    prev_end = end;
  }
  return FDY_OK;
}

extern "C" int fdy_layout_invert(const fdy_alloc* h_table, const uint64_t* h_new_base, uint32_t n_alloc,
                                 fdy_alloc* h_inv_table, uint64_t* h_inv_base, uint32_t* h_inv_region) {
  if (n_alloc == 0) return FDY_OK;
  if (!h_table || !h_new_base || !h_inv_table || !h_inv_base) return FDY_ERR_INVALID_ARG;
  if (fdy_table_validate(h_table, n_alloc, nullptr) != FDY_OK) return FDY_ERR_TABLE;
  std::vector<uint32_t> order(n_alloc);
  for (uint32_t r = 0; r < n_alloc; ++r) order[r] = r;
  std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
    return h_new_base[a] != h_new_base[b] ? h_new_base[a] < h_new_base[b] : a < b;
  });
  for (uint32_t k = 0; k < n_alloc; ++k) {
    const uint32_t r = order[k];
    h_inv_table[k].base = h_new_base[r];
    h_inv_table[k].size = h_table[r].size;
    h_inv_base[k] = h_table[r].base;
    if (h_inv_region) h_inv_region[k] = r;
  }
  // disjoint and non-wrapping in the new layout, or there is no way back
  return fdy_table_validate(h_inv_table, n_alloc, nullptr) == FDY_OK ? FDY_OK : FDY_ERR_TABLE;
}

extern "C" int fdy_layout_replay(const fdy_alloc* h_recorded, uint32_t n, uint64_t recorded_start,
                                 uint64_t new_start, uint64_t new_capacity, uint64_t new_used,
                                 uint64_t* h_new_base) {
  if (n == 0) return FDY_OK;
  if (!h_recorded || !h_new_base) return FDY_ERR_INVALID_ARG;
  if (fdy_table_validate(h_recorded, n, nullptr) != FDY_OK) return FDY_ERR_TABLE;
  if (h_recorded[0].base < recorded_start) return FDY_ERR_TABLE;
  if (h_recorded[0].base - recorded_start < new_used) return FDY_ERR_ORDER;
  // the table is valid, so the last allocation ends last and its end does not wrap
  const uint64_t end = h_recorded[n - 1].base + h_recorded[n - 1].size - recorded_start;
  if (end > new_capacity || new_start + end < new_start) return FDY_ERR_CAPACITY;
  for (uint32_t i = 0; i < n; ++i) h_new_base[i] = new_start + (h_recorded[i].base - recorded_start);
  return FDY_OK;
}

// ---- per-kernel event timing (bench support) -------------------------------------------
namespace {
struct ProfSlot {
  std::vector<hipEvent_t> a, b;
  int used = 0;
};
ProfSlot g_prof[FDY_PROF_SLOTS];
int g_prof_n = 0;
unsigned g_prof_mask = ~0u;
}  // namespace

void fdy::prof_begin(int slot, void* stream) {
  if (!g_prof_n || !((g_prof_mask >> slot) & 1u)) return;
  ProfSlot& s = g_prof[slot];
  if (s.used >= g_prof_n) return;
  (void)hipEventRecord(s.a[s.used], (hipStream_t)stream);
}

void fdy::prof_end(int slot, void* stream) {
  if (!g_prof_n || !((g_prof_mask >> slot) & 1u)) return;
  ProfSlot& s = g_prof[slot];
  if (s.used >= g_prof_n) return;
  (void)hipEventRecord(s.b[s.used], (hipStream_t)stream);
  ++s.used;
}

bool fdy::prof_take(int slot, void** start_event, void** stop_event) {
  if (!g_prof_n || !((g_prof_mask >> slot) & 1u)) return false;
  ProfSlot& s = g_prof[slot];
  if (s.used >= g_prof_n) return false;
  *start_event = (void*)s.a[s.used];
  *stop_event = (void*)s.b[s.used];
  ++s.used;
  return true;
}

extern "C" int fdy__prof_enable(int n_records) {
  for (auto& s : g_prof) {
    for (auto e : s.a) (void)hipEventDestroy(e);
    for (auto e : s.b) (void)hipEventDestroy(e);
    s.a.clear();
    s.b.clear();
    s.used = 0;
  }
  g_prof_n = 0;
  if (n_records <= 0) return 0;
  if (n_records > 4096) n_records = 4096;
  for (auto& s : g_prof) {
    s.a.resize(n_records);
    s.b.resize(n_records);
    for (int i = 0; i < n_records; ++i) {
      if (hipEventCreate(&s.a[i]) != hipSuccess || hipEventCreate(&s.b[i]) != hipSuccess) return -1;
    }
  }
  g_prof_n = n_records;
  return n_records;
}

extern "C" void fdy__prof_mask(unsigned mask) { g_prof_mask = mask; }

extern "C" int fdy__prof_read(int slot, int* n_records, float* total_ms, float* min_ms, float* max_ms) {
  if (slot < 0 || slot >= FDY_PROF_SLOTS) return -1;
  ProfSlot& s = g_prof[slot];
  float tot = 0.f, mn = 1e30f, mx = 0.f;
  for (int i = 0; i < s.used; ++i) {
    if (hipEventSynchronize(s.b[i]) != hipSuccess) return -1;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, s.a[i], s.b[i]) != hipSuccess) return -1;
    tot += ms;
    mn = ms < mn ? ms : mn;
    mx = ms > mx ? ms : mx;
  }
  if (n_records) *n_records = s.used;
  if (total_ms) *total_ms = tot;
  if (min_ms) *min_ms = s.used ? mn : 0.f;
  if (max_ms) *max_ms = mx;
  s.used = 0;
  return 0;
}

extern "C" const char* fdy__prof_name(int slot) {
  static const char* names[FDY_PROF_SLOTS] = {
      "scan_kernel", "scan_init_kernel", "reloc_segment_kernel", "fp_key_kernel", "fp_group_kernel",
      "mat_prep_graphs_kernel", "mat_prep_tiles_kernel", "mat_main_kernel", "scan_out_kernel",
      "scan_rebase_kernel", "scan_leafmap_kernel"};
  return slot >= 0 && slot < FDY_PROF_SLOTS ? names[slot] : "?";
}
