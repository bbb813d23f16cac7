/*
 * fdy_archive.h - binary on-disk form of a graph archive, C ABI.
 *
 * Section 5.3 of the paper (last paragraph) and Section 6.5 ("Composition of the archive"):
 * graph metadata (topology, node parameters, grouping manifest) is serialized in a binary
 * form because parsing a text form took seconds; 512 serialized graphs parse in under
 * 100 ms.  The paper gives no byte layout.  This one is made for the consumer: every section
 * is, byte for byte, one of the arrays that the calls of fdy.h take, so "parsing" is mapping
 * the file, checking the directory and (optionally) the contents, and the whole body goes to
 * the GPU in one copy; device pointers of the sections are the slab pointer plus fixed
 * offsets.  All integers are little-endian.
 *
 *   header (64 B)   0  char     magic[8]   "FDYARCH1"
 *                   8  uint32   version    1
 *                  12  uint32   n_sections (<= 64)
 *                  16  uint64   file_bytes
 *                  24  uint64   body_offset   multiple of 4096, >= 64 + 32 * n_sections
 *                  32  uint64   body_bytes    file_bytes - body_offset
 *                  40  uint64   head_sum      fdy_archive_sum of header (this field 0) + directory
 *                  48  uint64   reserved[2]   0
 *   directory      n_sections entries of 32 B, at byte 64:
 *                   0  uint32   kind          FDY_SEC_*, each kind at most once
 *                   4  uint32   elem_bytes    size of one element (fixed per kind)
 *                   8  uint64   offset        from the start of the file, multiple of 256,
 *                                             >= body_offset; entries ascending, no overlap
 *                  16  uint64   count         elements
 *                  24  uint64   sum           fdy_archive_sum of the section's bytes
 *   zero padding up to body_offset, then each section's bytes, each zero-padded to a
 *   multiple of 256 bytes; file_bytes is the end of the last section's padding.
 *
 * fdy_archive_sum(bytes, n): the bytes, zero-padded to a multiple of 8, read as 64-bit
 * words w[0..k): sum over i of w[i] * (2 i + 1), modulo 2^64.  (Every multiplier is odd, so
 * any change of a single word changes the sum; the sum guards against damage, not against
 * an adversary.)
 *
 * These are host-side calls; only fdy_archive_upload touches the GPU.  An open archive is
 * read-only and may be used from several threads.  Return codes are those of fdy.h.
 */
#ifndef FDY_ARCHIVE_H
#define FDY_ARCHIVE_H

#include <stddef.h>
#include <stdint.h>

#include "fdy.h"

#ifdef __cplusplus
extern "C" {
#endif

#define FDY_ARCHIVE_VERSION 1u
#define FDY_ARCHIVE_MAX_SECTIONS 64u

/* Section kinds.  S source graphs (the graphs whose blobs are stored: the templates, or
 * all captured graphs), T templates, G graphs, R ranks, A allocations. */
#define FDY_SEC_TABLE 1u      /* fdy_alloc[A]      allocation table of the captured layout  */
#define FDY_SEC_WORDS 2u      /* uint64[W]         argument blobs of the source graphs      */
#define FDY_SEC_WORD_OFF 3u   /* uint64[S+1]       first word of each source graph          */
#define FDY_SEC_NODES 4u      /* fdy_node[N]       node records of the source graphs        */
#define FDY_SEC_NODE_OFF 5u   /* uint64[S+1]                                                */
#define FDY_SEC_RELOCS 6u     /* fdy_reloc[K]      relocation table of WORDS                */
#define FDY_SEC_RELOC_OFF 7u  /* uint64[S+1]       first relocation of each source graph    */
#define FDY_SEC_GRAPH_TMPL 8u /* uint32[G]         grouping manifest: template of a graph   */
#define FDY_SEC_TMPL_GRAPH 9u /* uint32[T]         source graph that is template t          */
#define FDY_SEC_OVR 10u       /* fdy_ovr32[]       per-graph 32-bit overrides (may be empty) */
#define FDY_SEC_OVR_OFF 11u   /* uint64[G+1]                                                */
#define FDY_SEC_GOVR 12u      /* fdy_grid_ovr[]    per-graph grid overrides (may be empty)  */
#define FDY_SEC_GOVR_OFF 13u  /* uint64[G+1]                                                */
#define FDY_SEC_PATCH 14u     /* fdy_patch[]       per (template, rank) patches (optional)  */
#define FDY_SEC_PATCH_OFF 15u /* uint64[T*R+1]                                              */
#define FDY_SEC_KEYS 16u      /* uint64[G]         topology key of each graph (optional)    */
#define FDY_SEC_KIND_MAX 16u

/* Size in bytes of one element of a section kind (0 for an unknown kind). */
uint32_t fdy_archive_elem_bytes(uint32_t kind);

/* The checksum defined above over n bytes of host memory. */
uint64_t fdy_archive_sum(const void* h_bytes, size_t n);

/* One section to be written: `count` elements of `elem_bytes` each at host pointer `data`
 * (may be NULL when count is 0). */
typedef struct {
  uint32_t kind;
  uint32_t elem_bytes;
  uint64_t count;
  const void* data;
} fdy_archive_src;

/* Writes an archive with the given sections, in the given order, to `path` (created or
 * replaced).  The container rules are enforced (known kinds, each at most once, elem_bytes
 * matching the kind); the contents are not interpreted.
 * FDY_ERR_INVALID_ARG: null pointers, n_sections > FDY_ARCHIVE_MAX_SECTIONS, unknown or
 * repeated kind, wrong elem_bytes; FDY_ERR_IO: the file could not be created or written
 * (a partial file is removed). */
int fdy_archive_write(const char* path, const fdy_archive_src* h_sections, uint32_t n_sections);

typedef struct fdy_archive fdy_archive; /* opaque; owns a read-only mapping of the file */

#define FDY_ARCHIVE_VERIFY_SUMS 1u /* also recompute every section's sum at open */

/* Maps the file and checks the container: magic, version, sizes against the real file
 * size, head_sum, directory rules (known kinds once each, element sizes, alignment, order,
 * bounds), zero reserved fields; with FDY_ARCHIVE_VERIFY_SUMS every section's sum.
 * FDY_ERR_IO: cannot open / map; FDY_ERR_FORMAT: not an archive or a damaged container;
 * FDY_ERR_CHECKSUM: a sum does not match.  On error *out is NULL. */
int fdy_archive_open(const char* path, uint32_t flags, fdy_archive** out);
int fdy_archive_close(fdy_archive* a);

/* Text describing what the last failing fdy_archive_* call on this thread found ("" if
 * none). */
const char* fdy_archive_last_failure(void);

uint32_t fdy_archive_section_count(const fdy_archive* a);
uint64_t fdy_archive_file_bytes(const fdy_archive* a);
uint64_t fdy_archive_body_bytes(const fdy_archive* a);

/* Host view of a section: pointer into the mapping (valid until close, 256-byte aligned),
 * element count and size.  Output pointers may be NULL.  FDY_ERR_INVALID_ARG if the archive
 * has no section of that kind. */
int fdy_archive_section(const fdy_archive* a, uint32_t kind, const void** h_data, uint64_t* count,
                        uint32_t* elem_bytes);

/* What fdy_archive_check found out about the archive. */
typedef struct {
  uint32_t n_src_graphs; /* S */
  uint32_t n_templates;  /* T */
  uint32_t n_graphs;     /* G */
  uint32_t n_ranks;      /* R (0: no patch sections) */
  uint32_t n_alloc;      /* A */
  uint32_t reserved;
  uint64_t n_words;      /* W */
  uint64_t n_nodes;      /* N */
  uint64_t n_relocs;     /* K */
  uint64_t out_words_per_map; /* sum over graphs of the word count of their template */
  uint64_t out_nodes_total;   /* sum over graphs of the node count of their template */
} fdy_archive_info;

/* Checks that the sections describe a consistent archive, i.e. one that fdy_materialize
 * accepts (the rules of fdy_mat_desc in fdy.h) and that fdy_scan_pointers could have
 * produced:
 *   - every section except PATCH, PATCH_OFF and KEYS is present (a list may be empty, its
 *     offsets are then all 0); PATCH and PATCH_OFF come as a pair;
 *   - the table is valid per fdy_table_validate; A, S, T, G >= 1 and within fdy.h's limits;
 *   - every offset array starts at 0, never decreases, ends at the count of its data
 *     section and has the length stated above (R = (count - 1) / T must be whole, >= 1);
 *   - every node's blob_len is a multiple of 8 and the blob lengths of a source graph add
 *     up to its word count times 8; W < 2^32;
 *   - relocations of source graph s have strictly ascending `word` inside the graph's word
 *     range, region < A, offset < size of the region, and WORDS[word] equals
 *     base[region] + offset;
 *   - graph_tmpl[g] < T; tmpl_graph[t] < S;
 *   - overrides of graph g: byte_off strictly ascending, multiple of 4, inside the
 *     template's blob; grid overrides: node strictly ascending, inside the template's
 *     nodes; patches of (t, r): word strictly ascending inside template t, reserved 0;
 *   - KEYS, if present, has G entries, and two graphs have equal keys exactly if they have
 *     the same template.
 * FDY_OK, or FDY_ERR_CONTENT with the first violated rule in fdy_archive_last_failure().
 * `out` may be NULL. */
int fdy_archive_check(const fdy_archive* a, fdy_archive_info* out);

/* Copies the body (every section, with padding) to device memory: d_slab must be 256-byte
 * aligned and hold fdy_archive_body_bytes(a).  Asynchronous on `hip_stream` as far as a
 * copy from pageable host memory is; the mapping must stay open until the stream has
 * passed the copy.  FDY_ERR_HIP if the copy fails. */
int fdy_archive_upload(const fdy_archive* a, void* d_slab, size_t slab_bytes, void* hip_stream);

/* Device address of a section inside a slab filled by fdy_archive_upload (pointer
 * arithmetic only; NULL for an absent or empty section). */
const void* fdy_archive_device_section(const fdy_archive* a, uint32_t kind, const void* d_slab);

/* Fills the archive-side fields of a materialize descriptor from an archive that passed
 * fdy_archive_check, with device pointers into `d_slab`: the S/T/G/A/R scalars, the totals,
 * and every source, manifest, override and patch array.  The load-side fields (n_maps,
 * new_base, map_rank) are left untouched for the caller; n_ranks is R only once the caller
 * sets map_rank, so it is written as R and the caller zeroes it to ignore patches.
 * FDY_ERR_CONTENT if the archive fails the check. */
int fdy_archive_mat_desc(const fdy_archive* a, const void* d_slab, fdy_mat_desc* h_desc);

#ifdef __cplusplus
}
#endif
#endif /* FDY_ARCHIVE_H */
