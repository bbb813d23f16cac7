// fdy_archive.hip - binary on-disk form of a graph archive (host code; one device copy).
//
// Section 5.3 (last paragraph) and Section 6.5 of the paper: graph metadata is serialized in
// a binary form so that 512 graphs parse in under 100 ms.  Every section of this format is
// one of the arrays the device calls take, so opening is a mapping plus a directory check,
// the content check is a handful of linear passes, and the body goes to the GPU in one copy.
#include <hip/hip_runtime.h>

#include <errno.h>
#include <fcntl.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <new>
#include <utility>
#include <vector>

#include "fdy_archive.h"

namespace {

constexpr uint64_t kHeaderBytes = 64, kDirEntryBytes = 32, kBodyAlign = 4096, kSectionAlign = 256;
const char kMagic[8] = {'F', 'D', 'Y', 'A', 'R', 'C', 'H', '1'};

struct Header {
  char magic[8];
  uint32_t version, n_sections;
  uint64_t file_bytes, body_offset, body_bytes, head_sum, reserved[2];
};
static_assert(sizeof(Header) == kHeaderBytes, "header layout");

struct DirEntry {
  uint32_t kind, elem_bytes;
  uint64_t offset, count, sum;
};
static_assert(sizeof(DirEntry) == kDirEntryBytes, "directory layout");

thread_local char g_failure[256] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_failure, sizeof g_failure, fmt, ap);
  va_end(ap);
  return code;
}

uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

const char* kind_name(uint32_t kind) {
  static const char* names[FDY_SEC_KIND_MAX + 1] = {
      "?",       "TABLE",      "WORDS",      "WORD_OFF", "NODES",   "NODE_OFF", "RELOCS", "RELOC_OFF", "GRAPH_TMPL",
      "TMPL_GRAPH", "OVR",     "OVR_OFF",    "GOVR",     "GOVR_OFF", "PATCH",   "PATCH_OFF", "KEYS"};
  return kind <= FDY_SEC_KIND_MAX ? names[kind] : "?";
}

}  // namespace

struct fdy_archive {
  const unsigned char* map = nullptr;
  uint64_t bytes = 0;
  Header head{};
  DirEntry dir[FDY_ARCHIVE_MAX_SECTIONS];
  int slot[FDY_SEC_KIND_MAX + 1];  // directory index of each kind, -1 if absent
};

extern "C" uint32_t fdy_archive_elem_bytes(uint32_t kind) {
  switch (kind) {
    case FDY_SEC_TABLE: return sizeof(fdy_alloc);
    case FDY_SEC_NODES: return sizeof(fdy_node);
    case FDY_SEC_RELOCS: return sizeof(fdy_reloc);
    case FDY_SEC_OVR: return sizeof(fdy_ovr32);
    case FDY_SEC_GOVR: return sizeof(fdy_grid_ovr);
    case FDY_SEC_PATCH: return sizeof(fdy_patch);
    case FDY_SEC_GRAPH_TMPL:
    case FDY_SEC_TMPL_GRAPH: return 4;
    case FDY_SEC_WORDS:
    case FDY_SEC_WORD_OFF:
    case FDY_SEC_NODE_OFF:
    case FDY_SEC_RELOC_OFF:
    case FDY_SEC_OVR_OFF:
    case FDY_SEC_GOVR_OFF:
    case FDY_SEC_PATCH_OFF:
    case FDY_SEC_KEYS: return 8;
    default: return 0;
  }
}

extern "C" uint64_t fdy_archive_sum(const void* h_bytes, size_t n) {
  const unsigned char* p = static_cast<const unsigned char*>(h_bytes);
  const size_t k = n / 8;
  // four independent accumulators keep the multiplier pipeline full
  uint64_t s0 = 0, s1 = 0, s2 = 0, s3 = 0;
  size_t i = 0;
  for (; i + 4 <= k; i += 4) {
    uint64_t w[4];
    memcpy(w, p + i * 8, 32);
    s0 += w[0] * (2 * (uint64_t)i + 1);
    s1 += w[1] * (2 * (uint64_t)i + 3);
    s2 += w[2] * (2 * (uint64_t)i + 5);
    s3 += w[3] * (2 * (uint64_t)i + 7);
  }
  for (; i < k; ++i) {
    uint64_t w;
    memcpy(&w, p + i * 8, 8);
    s0 += w * (2 * (uint64_t)i + 1);
  }
  if (n % 8) {
    uint64_t w = 0;
    memcpy(&w, p + k * 8, n % 8);
    s0 += w * (2 * (uint64_t)k + 1);
  }
  return s0 + s1 + s2 + s3;
}

namespace {

// Shared by the writer and the reader: the container rules of a directory whose offsets are
// already assigned.  Returns nullptr or a description of the first violated rule.
const char* directory_violation(const Header& h, const DirEntry* dir) {
  static thread_local char text[160];
  if (h.n_sections > FDY_ARCHIVE_MAX_SECTIONS) return "too many sections";
  if (h.body_offset % kBodyAlign || h.body_offset < kHeaderBytes + kDirEntryBytes * h.n_sections)
    return "body offset misaligned or inside the directory";
  if (h.body_offset > h.file_bytes || h.body_bytes != h.file_bytes - h.body_offset)
    return "body size does not match the file size";
  if (h.reserved[0] || h.reserved[1]) return "reserved header field not zero";
  bool seen[FDY_SEC_KIND_MAX + 1] = {};
  uint64_t cursor = h.body_offset;
  for (uint32_t i = 0; i < h.n_sections; ++i) {
    const DirEntry& e = dir[i];
    const uint32_t eb = fdy_archive_elem_bytes(e.kind);
    if (!eb) {
      snprintf(text, sizeof text, "directory entry %u: unknown kind %u", i, e.kind);
      return text;
    }
    if (seen[e.kind]) {
      snprintf(text, sizeof text, "section %s appears twice", kind_name(e.kind));
      return text;
    }
    seen[e.kind] = true;
    if (e.elem_bytes != eb) {
      snprintf(text, sizeof text, "section %s: element size %u, expected %u", kind_name(e.kind), e.elem_bytes, eb);
      return text;
    }
    if (e.offset % kSectionAlign || e.offset < cursor) {
      snprintf(text, sizeof text, "section %s: offset misaligned, out of order or overlapping", kind_name(e.kind));
      return text;
    }
    if (e.count > (UINT64_MAX - kSectionAlign) / eb || e.offset > h.file_bytes ||
        round_up(e.count * eb, kSectionAlign) > h.file_bytes - e.offset) {
      snprintf(text, sizeof text, "section %s: extends past the end of the file", kind_name(e.kind));
      return text;
    }
    cursor = e.offset + round_up(e.count * eb, kSectionAlign);
  }
  if (cursor != h.file_bytes) return "file size does not end at the last section";
  return nullptr;
}

uint64_t head_sum_of(Header h, const DirEntry* dir) {
  h.head_sum = 0;
  std::vector<unsigned char> buf(kHeaderBytes + kDirEntryBytes * h.n_sections);
  memcpy(buf.data(), &h, kHeaderBytes);
  if (h.n_sections) memcpy(buf.data() + kHeaderBytes, dir, kDirEntryBytes * h.n_sections);
  return fdy_archive_sum(buf.data(), buf.size());
}

bool write_all(int fd, const void* data, size_t n) {
  const unsigned char* p = static_cast<const unsigned char*>(data);
  while (n) {
    const ssize_t w = write(fd, p, n > (1u << 30) ? (1u << 30) : n);
    if (w < 0) {
      if (errno == EINTR) continue;
      return false;
    }
    p += w;
    n -= (size_t)w;
  }
  return true;
}

bool write_zeros(int fd, uint64_t n) {
  static const unsigned char zeros[4096] = {};
  while (n) {
    const size_t c = n > sizeof zeros ? sizeof zeros : (size_t)n;
    if (!write_all(fd, zeros, c)) return false;
    n -= c;
  }
  return true;
}

}  // namespace

extern "C" int fdy_archive_write(const char* path, const fdy_archive_src* secs, uint32_t n) {
  g_failure[0] = 0;
  if (!path || (n && !secs)) return fail(FDY_ERR_INVALID_ARG, "null argument");
  if (n > FDY_ARCHIVE_MAX_SECTIONS) return fail(FDY_ERR_INVALID_ARG, "more than %u sections", FDY_ARCHIVE_MAX_SECTIONS);
  Header h{};
  memcpy(h.magic, kMagic, 8);
  h.version = FDY_ARCHIVE_VERSION;
  h.n_sections = n;
  h.body_offset = round_up(kHeaderBytes + kDirEntryBytes * n, kBodyAlign);
  DirEntry dir[FDY_ARCHIVE_MAX_SECTIONS];
  memset(dir, 0, sizeof dir);
  uint64_t cursor = h.body_offset;
  for (uint32_t i = 0; i < n; ++i) {
    const uint32_t eb = fdy_archive_elem_bytes(secs[i].kind);
    if (!eb || secs[i].elem_bytes != eb)
      return fail(FDY_ERR_INVALID_ARG, "section %u: unknown kind %u or element size %u", i, secs[i].kind,
                  secs[i].elem_bytes);
    if (secs[i].count && !secs[i].data) return fail(FDY_ERR_INVALID_ARG, "section %u: null data", i);
    if (secs[i].count > (UINT64_MAX >> 8) / eb) return fail(FDY_ERR_INVALID_ARG, "section %u: count out of range", i);
    for (uint32_t j = 0; j < i; ++j)
      if (secs[j].kind == secs[i].kind)
        return fail(FDY_ERR_INVALID_ARG, "section %s given twice", kind_name(secs[i].kind));
    dir[i].kind = secs[i].kind;
    dir[i].elem_bytes = eb;
    dir[i].offset = cursor;
    dir[i].count = secs[i].count;
    dir[i].sum = fdy_archive_sum(secs[i].data, (size_t)(secs[i].count * eb));
    cursor += round_up(secs[i].count * eb, kSectionAlign);
  }
  h.file_bytes = cursor;
  h.body_bytes = cursor - h.body_offset;
  h.head_sum = head_sum_of(h, dir);

  const int fd = open(path, O_WRONLY | O_CREAT | O_TRUNC | O_CLOEXEC, 0644);
  if (fd < 0) return fail(FDY_ERR_IO, "cannot create %s: %s", path, strerror(errno));
  bool ok = write_all(fd, &h, kHeaderBytes) && write_all(fd, dir, kDirEntryBytes * n) &&
            write_zeros(fd, h.body_offset - kHeaderBytes - kDirEntryBytes * n);
  for (uint32_t i = 0; ok && i < n; ++i) {
    const uint64_t nb = secs[i].count * dir[i].elem_bytes;
    ok = write_all(fd, secs[i].data, (size_t)nb) && write_zeros(fd, round_up(nb, kSectionAlign) - nb);
  }
  const int saved = errno;
  if (close(fd) != 0) ok = false;
  if (!ok) {
    unlink(path);
    return fail(FDY_ERR_IO, "cannot write %s: %s", path, strerror(saved ? saved : errno));
  }
  return FDY_OK;
}

extern "C" int fdy_archive_close(fdy_archive* a) {
  if (!a) return FDY_OK;
  int rc = FDY_OK;
  if (a->map && munmap(const_cast<unsigned char*>(a->map), (size_t)a->bytes) != 0) rc = FDY_ERR_IO;
  delete a;
  return rc;
}

extern "C" int fdy_archive_open(const char* path, uint32_t flags, fdy_archive** out) {
  g_failure[0] = 0;
  if (out) *out = nullptr;
  if (!path || !out || (flags & ~FDY_ARCHIVE_VERIFY_SUMS)) return fail(FDY_ERR_INVALID_ARG, "null argument or unknown flag");
  const int fd = open(path, O_RDONLY | O_CLOEXEC);
  if (fd < 0) return fail(FDY_ERR_IO, "cannot open %s: %s", path, strerror(errno));
  struct stat st;
  if (fstat(fd, &st) != 0 || !S_ISREG(st.st_mode)) {
    close(fd);
    return fail(FDY_ERR_IO, "%s is not a regular file", path);
  }
  const uint64_t bytes = (uint64_t)st.st_size;
  if (bytes < kHeaderBytes) {
    close(fd);
    return fail(FDY_ERR_FORMAT, "file shorter than an archive header");
  }
  void* m = mmap(nullptr, (size_t)bytes, PROT_READ, MAP_PRIVATE, fd, 0);
  const int map_errno = errno;
  close(fd);
  if (m == MAP_FAILED) return fail(FDY_ERR_IO, "cannot map %s: %s", path, strerror(map_errno));
  fdy_archive* a = new (std::nothrow) fdy_archive;
  if (!a) {
    munmap(m, (size_t)bytes);
    return fail(FDY_ERR_IO, "out of memory");
  }
  a->map = static_cast<const unsigned char*>(m);
  a->bytes = bytes;
  auto reject = [&](int code, const char* what) {
    fdy_archive_close(a);
    return fail(code, "%s", what);
  };
  memcpy(&a->head, a->map, kHeaderBytes);
  const Header& h = a->head;
  if (memcmp(h.magic, kMagic, 8) != 0) return reject(FDY_ERR_FORMAT, "magic bytes do not match");
  if (h.version != FDY_ARCHIVE_VERSION) return reject(FDY_ERR_FORMAT, "unsupported format version");
  if (h.file_bytes != bytes) return reject(FDY_ERR_FORMAT, "stored file size differs from the real one (truncated?)");
  if (h.n_sections > FDY_ARCHIVE_MAX_SECTIONS || kHeaderBytes + kDirEntryBytes * h.n_sections > bytes)
    return reject(FDY_ERR_FORMAT, "section count out of range");
  memcpy(a->dir, a->map + kHeaderBytes, kDirEntryBytes * h.n_sections);
  if (const char* v = directory_violation(h, a->dir)) return reject(FDY_ERR_FORMAT, v);
  if (head_sum_of(h, a->dir) != h.head_sum) return reject(FDY_ERR_CHECKSUM, "header and directory sum does not match");
  for (int& s : a->slot) s = -1;
  for (uint32_t i = 0; i < h.n_sections; ++i) a->slot[a->dir[i].kind] = (int)i;
  if (flags & FDY_ARCHIVE_VERIFY_SUMS) {
    for (uint32_t i = 0; i < h.n_sections; ++i) {
      const DirEntry& e = a->dir[i];
      if (fdy_archive_sum(a->map + e.offset, (size_t)(e.count * e.elem_bytes)) != e.sum) {
        char text[96];
        snprintf(text, sizeof text, "section %s: sum does not match", kind_name(e.kind));
        return reject(FDY_ERR_CHECKSUM, text);
      }
    }
  }
  *out = a;
  return FDY_OK;
}

extern "C" const char* fdy_archive_last_failure(void) { return g_failure; }
extern "C" uint32_t fdy_archive_section_count(const fdy_archive* a) { return a ? a->head.n_sections : 0; }
extern "C" uint64_t fdy_archive_file_bytes(const fdy_archive* a) { return a ? a->bytes : 0; }
extern "C" uint64_t fdy_archive_body_bytes(const fdy_archive* a) { return a ? a->head.body_bytes : 0; }

extern "C" int fdy_archive_section(const fdy_archive* a, uint32_t kind, const void** h_data, uint64_t* count,
                                   uint32_t* elem_bytes) {
  if (h_data) *h_data = nullptr;
  if (count) *count = 0;
  if (elem_bytes) *elem_bytes = 0;
  if (!a || kind == 0 || kind > FDY_SEC_KIND_MAX || a->slot[kind] < 0) return FDY_ERR_INVALID_ARG;
  const DirEntry& e = a->dir[a->slot[kind]];
  if (h_data) *h_data = a->map + e.offset;
  if (count) *count = e.count;
  if (elem_bytes) *elem_bytes = e.elem_bytes;
  return FDY_OK;
}

namespace {

template <typename T>
struct View {
  const T* p = nullptr;
  uint64_t n = 0;
  bool present = false;
  const T& operator[](uint64_t i) const { return p[i]; }
};

template <typename T>
View<T> view(const fdy_archive* a, uint32_t kind) {
  View<T> v;
  const void* p = nullptr;
  if (fdy_archive_section(a, kind, &p, &v.n, nullptr) == FDY_OK) {
    v.p = static_cast<const T*>(p);
    v.present = true;
  }
  return v;
}

// offsets: `len` entries, from 0, never decreasing, ending at `total`
const char* offsets_violation(const View<uint64_t>& off, uint64_t len, uint64_t total) {
  if (off.n != len) return "has the wrong length";
  if (off[0] != 0) return "does not start at 0";
  for (uint64_t i = 1; i < len; ++i)
    if (off[i] < off[i - 1]) return "decreases";
  if (off[len - 1] != total) return "does not end at the size of its data section";
  return nullptr;
}

int content_check(const fdy_archive* a, fdy_archive_info* out) {
  const auto bad = [](const char* fmt, auto... args) { return fail(FDY_ERR_CONTENT, fmt, args...); };
  const auto table = view<fdy_alloc>(a, FDY_SEC_TABLE);
  const auto words = view<uint64_t>(a, FDY_SEC_WORDS);
  const auto word_off = view<uint64_t>(a, FDY_SEC_WORD_OFF);
  const auto nodes = view<fdy_node>(a, FDY_SEC_NODES);
  const auto node_off = view<uint64_t>(a, FDY_SEC_NODE_OFF);
  const auto relocs = view<fdy_reloc>(a, FDY_SEC_RELOCS);
  const auto reloc_off = view<uint64_t>(a, FDY_SEC_RELOC_OFF);
  const auto graph_tmpl = view<uint32_t>(a, FDY_SEC_GRAPH_TMPL);
  const auto tmpl_graph = view<uint32_t>(a, FDY_SEC_TMPL_GRAPH);
  const auto ovr = view<fdy_ovr32>(a, FDY_SEC_OVR);
  const auto ovr_off = view<uint64_t>(a, FDY_SEC_OVR_OFF);
  const auto govr = view<fdy_grid_ovr>(a, FDY_SEC_GOVR);
  const auto govr_off = view<uint64_t>(a, FDY_SEC_GOVR_OFF);
  const auto patch = view<fdy_patch>(a, FDY_SEC_PATCH);
  const auto patch_off = view<uint64_t>(a, FDY_SEC_PATCH_OFF);
  const auto keys = view<uint64_t>(a, FDY_SEC_KEYS);

  if (!table.present || !words.present || !word_off.present || !nodes.present || !node_off.present ||
      !relocs.present || !reloc_off.present || !graph_tmpl.present || !tmpl_graph.present || !ovr.present ||
      !ovr_off.present || !govr.present || !govr_off.present)
    return bad("a required section is missing");
  if (patch.present != patch_off.present) return bad("PATCH is present without PATCH_OFF, or the reverse");

  constexpr uint64_t kMaxGraphs = 1u << 20;
  if (table.n < 1 || table.n > 0xffffffffu) return bad("TABLE: allocation count out of range");
  uint32_t bad_index = 0;
  if (fdy_table_validate(table.p, (uint32_t)table.n, &bad_index) != FDY_OK)
    return bad("TABLE: entry %u breaks the order / overlap / size rules", bad_index);
  if (word_off.n < 2 || word_off.n - 1 > kMaxGraphs) return bad("WORD_OFF: source graph count out of range");
  const uint64_t S = word_off.n - 1, T = tmpl_graph.n, G = graph_tmpl.n, A = table.n;
  if (T < 1 || T > kMaxGraphs || G < 1 || G > kMaxGraphs) return bad("manifest: template or graph count out of range");
  if (words.n >> 32) return bad("WORDS: 2^32 words or more");
  if (const char* v = offsets_violation(word_off, S + 1, words.n)) return bad("WORD_OFF %s", v);
  if (const char* v = offsets_violation(node_off, S + 1, nodes.n)) return bad("NODE_OFF %s", v);
  if (const char* v = offsets_violation(reloc_off, S + 1, relocs.n)) return bad("RELOC_OFF %s", v);

  for (uint64_t s = 0; s < S; ++s) {
    uint64_t blob_bytes = 0;
    for (uint64_t i = node_off[s]; i < node_off[s + 1]; ++i) {
      if (nodes[i].blob_len % 8) return bad("NODES: node %llu has a blob length that is not a multiple of 8", (unsigned long long)i);
      blob_bytes += nodes[i].blob_len;
    }
    if (blob_bytes != (word_off[s + 1] - word_off[s]) * 8)
      return bad("source graph %llu: blob lengths of its nodes do not add up to its words", (unsigned long long)s);
    const uint64_t w_lo = word_off[s], w_hi = word_off[s + 1];
    uint64_t prev = 0;
    for (uint64_t i = reloc_off[s]; i < reloc_off[s + 1]; ++i) {
      const fdy_reloc& r = relocs[i];
      if (r.word < w_lo || r.word >= w_hi || (i > reloc_off[s] && r.word <= prev))
        return bad("RELOCS: entry %llu is outside its graph's words or not ascending", (unsigned long long)i);
      prev = r.word;
      if (r.region >= A || r.offset >= table[r.region].size)
        return bad("RELOCS: entry %llu names a region or offset outside the table", (unsigned long long)i);
      if (words[r.word] != table[r.region].base + r.offset)
        return bad("RELOCS: entry %llu does not match the word it describes", (unsigned long long)i);
    }
  }

  for (uint64_t t = 0; t < T; ++t)
    if (tmpl_graph[t] >= S) return bad("TMPL_GRAPH: template %llu names a source graph that is not stored", (unsigned long long)t);
  uint64_t out_words = 0, out_nodes = 0;
  for (uint64_t g = 0; g < G; ++g) {
    if (graph_tmpl[g] >= T) return bad("GRAPH_TMPL: graph %llu names a template that does not exist", (unsigned long long)g);
    const uint64_t s = tmpl_graph[graph_tmpl[g]];
    out_words += word_off[s + 1] - word_off[s];
    out_nodes += node_off[s + 1] - node_off[s];
  }

  {
    if (const char* v = offsets_violation(ovr_off, G + 1, ovr.n)) return bad("OVR_OFF %s", v);
    for (uint64_t g = 0; g < G; ++g) {
      const uint64_t s = tmpl_graph[graph_tmpl[g]];
      const uint64_t blob = (word_off[s + 1] - word_off[s]) * 8;
      for (uint64_t i = ovr_off[g]; i < ovr_off[g + 1]; ++i)
        if (ovr[i].byte_off % 4 || ovr[i].byte_off >= blob || (i > ovr_off[g] && ovr[i].byte_off <= ovr[i - 1].byte_off))
          return bad("OVR: entry %llu is misaligned, outside the blob or not ascending", (unsigned long long)i);
    }
  }
  {
    if (const char* v = offsets_violation(govr_off, G + 1, govr.n)) return bad("GOVR_OFF %s", v);
    for (uint64_t g = 0; g < G; ++g) {
      const uint64_t s = tmpl_graph[graph_tmpl[g]];
      const uint64_t nn = node_off[s + 1] - node_off[s];
      for (uint64_t i = govr_off[g]; i < govr_off[g + 1]; ++i)
        if (govr[i].node >= nn || (i > govr_off[g] && govr[i].node <= govr[i - 1].node))
          return bad("GOVR: entry %llu is outside the graph's nodes or not ascending", (unsigned long long)i);
    }
  }
  uint64_t R = 0;
  if (patch.present) {
    if (patch_off.n < 2 || (patch_off.n - 1) % T) return bad("PATCH_OFF has the wrong length");
    R = (patch_off.n - 1) / T;
    if (R > 0xffffu) return bad("PATCH_OFF: rank count out of range");
    if (const char* v = offsets_violation(patch_off, T * R + 1, patch.n)) return bad("PATCH_OFF %s", v);
    for (uint64_t t = 0; t < T; ++t) {
      const uint64_t s = tmpl_graph[t];
      const uint64_t nw = word_off[s + 1] - word_off[s];
      for (uint64_t r = 0; r < R; ++r) {
        const uint64_t lo = patch_off[t * R + r], hi = patch_off[t * R + r + 1];
        for (uint64_t i = lo; i < hi; ++i)
          if (patch[i].word >= nw || patch[i].reserved || (i > lo && patch[i].word <= patch[i - 1].word))
            return bad("PATCH: entry %llu is outside the template, not ascending or has a nonzero reserved field",
                       (unsigned long long)i);
      }
    }
  }
  if (keys.present) {
    if (keys.n != G) return bad("KEYS has the wrong length");
    // equal keys exactly for equal templates: sorted by key, a key must not change template,
    // and sorted by template, a template must not change key
    std::vector<std::pair<uint64_t, uint32_t>> kt(G);
    for (uint64_t g = 0; g < G; ++g) kt[g] = {keys[g], graph_tmpl[g]};
    std::sort(kt.begin(), kt.end());
    for (uint64_t g = 1; g < G; ++g)
      if (kt[g].first == kt[g - 1].first && kt[g].second != kt[g - 1].second)
        return bad("KEYS: one key is shared by two templates");
    std::vector<uint64_t> key_of(T, 0);
    std::vector<char> have(T, 0);
    for (uint64_t g = 0; g < G; ++g) {
      const uint32_t t = graph_tmpl[g];
      if (have[t] && key_of[t] != keys[g]) return bad("KEYS: one template has two keys");
      have[t] = 1;
      key_of[t] = keys[g];
    }
  }
  if (out) {
    memset(out, 0, sizeof *out);
    out->n_src_graphs = (uint32_t)S;
    out->n_templates = (uint32_t)T;
    out->n_graphs = (uint32_t)G;
    out->n_ranks = (uint32_t)R;
    out->n_alloc = (uint32_t)A;
    out->n_words = words.n;
    out->n_nodes = nodes.n;
    out->n_relocs = relocs.n;
    out->out_words_per_map = out_words;
    out->out_nodes_total = out_nodes;
  }
  return FDY_OK;
}

}  // namespace

extern "C" int fdy_archive_check(const fdy_archive* a, fdy_archive_info* out) {
  g_failure[0] = 0;
  if (!a) return fail(FDY_ERR_INVALID_ARG, "null archive");
  return content_check(a, out);
}

extern "C" int fdy_archive_upload(const fdy_archive* a, void* d_slab, size_t slab_bytes, void* hip_stream) {
  g_failure[0] = 0;
  if (!a || (!d_slab && a->head.body_bytes) || (uintptr_t)d_slab % kSectionAlign || slab_bytes < a->head.body_bytes)
    return fail(FDY_ERR_INVALID_ARG, "null archive, or slab null, misaligned or too small");
  if (!a->head.body_bytes) return FDY_OK;
  const hipError_t e = hipMemcpyAsync(d_slab, a->map + a->head.body_offset, (size_t)a->head.body_bytes,
                                      hipMemcpyHostToDevice, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(FDY_ERR_HIP, "hipMemcpyAsync: %s", hipGetErrorString(e));
  }
  return FDY_OK;
}

extern "C" const void* fdy_archive_device_section(const fdy_archive* a, uint32_t kind, const void* d_slab) {
  if (!a || !d_slab || kind == 0 || kind > FDY_SEC_KIND_MAX || a->slot[kind] < 0) return nullptr;
  const DirEntry& e = a->dir[a->slot[kind]];
  if (!e.count) return nullptr;
  return static_cast<const unsigned char*>(d_slab) + (e.offset - a->head.body_offset);
}

extern "C" int fdy_archive_mat_desc(const fdy_archive* a, const void* d_slab, fdy_mat_desc* d) {
  g_failure[0] = 0;
  if (!a || !d_slab || !d) return fail(FDY_ERR_INVALID_ARG, "null argument");
  fdy_archive_info info;
  const int rc = content_check(a, &info);
  if (rc != FDY_OK) return rc;
  d->n_src_graphs = info.n_src_graphs;
  d->n_templates = info.n_templates;
  d->n_graphs = info.n_graphs;
  d->n_alloc = info.n_alloc;
  d->n_ranks = info.n_ranks;
  d->out_words_per_map = info.out_words_per_map;
  d->out_nodes_total = info.out_nodes_total;
  const auto at = [&](uint32_t kind) { return fdy_archive_device_section(a, kind, d_slab); };
  d->src_words = static_cast<const uint64_t*>(at(FDY_SEC_WORDS));
  d->src_word_off = static_cast<const uint64_t*>(at(FDY_SEC_WORD_OFF));
  d->src_nodes = static_cast<const fdy_node*>(at(FDY_SEC_NODES));
  d->src_node_off = static_cast<const uint64_t*>(at(FDY_SEC_NODE_OFF));
  d->relocs = static_cast<const fdy_reloc*>(at(FDY_SEC_RELOCS));
  d->src_reloc_off = static_cast<const uint64_t*>(at(FDY_SEC_RELOC_OFF));
  d->tmpl_graph = static_cast<const uint32_t*>(at(FDY_SEC_TMPL_GRAPH));
  d->graph_tmpl = static_cast<const uint32_t*>(at(FDY_SEC_GRAPH_TMPL));
  d->ovr = static_cast<const fdy_ovr32*>(at(FDY_SEC_OVR));
  d->ovr_off = static_cast<const uint64_t*>(at(FDY_SEC_OVR_OFF));
  d->govr = static_cast<const fdy_grid_ovr*>(at(FDY_SEC_GOVR));
  d->govr_off = static_cast<const uint64_t*>(at(FDY_SEC_GOVR_OFF));
  d->patch = static_cast<const fdy_patch*>(at(FDY_SEC_PATCH));
  d->patch_off = static_cast<const uint64_t*>(at(FDY_SEC_PATCH_OFF));
  return FDY_OK;
}
