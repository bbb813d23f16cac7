/*
 * fdy.h - C ABI of the graph-context materialization core for MI355X (gfx950).
 *
 * The library turns the per-graph "parameter preparation" that the paper runs on
 * CPU worker threads at LOAD time (Section 4.2.1, "Topology-based Intra-Rank Graph
 * Grouping") into one-GPU data transforms, and relaxes the paper's identical-layout
 * requirement (Section 4.1.1, "Deterministic Memory Layout"): when a new instance
 * cannot be given the capture run's base addresses, every pointer embedded in the
 * captured kernel-argument buffers is found by interval membership against the
 * allocation table that the deterministic allocator records, and rebased.  The scan
 * is kernel-agnostic on purpose: argument buffers are opaque byte arrays that may
 * hide pointers inside library-private structs (Section 2.2; Appendix B shows one
 * such 1720-byte buffer).
 *
 * Conventions that hold for every entry point
 *  - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The caller owns
 *    every buffer; the library never allocates or frees device memory and copies nothing
 *    between host and device.  State between calls lives in buffers of the caller's (a
 *    prepared table, see fdy_scan_table_prepare), with one exception: the process-wide
 *    tuning knobs and timing records declared in fdy_internal.h (measurement support, off
 *    and at their defaults unless a caller touches them; not thread-safe).
 *  - Every call that takes a stream only ENQUEUES kernels on it (hipStream_t passed as
 *    void*; NULL = the default stream).  Outputs are valid once the caller has
 *    synchronized that stream.  Calls on one stream may be chained without host syncs:
 *    device scalars produced by one call (reloc count, template count) are consumed by
 *    the next from device memory.
 *  - Return value: FDY_OK (0) or a negative FDY_ERR_* for errors the host can see
 *    (null or misaligned pointers, sizes out of range, workspace too small, a failed
 *    launch).  Errors only the device can see (an index out of range inside a device
 *    table, more relocation hits than capacity) never cause an out-of-bounds access:
 *    the offending entry is skipped and a FDY_ST_* bit is OR-ed into *d_status
 *    (a device uint32_t the caller zeroes beforehand and reads after synchronizing;
 *    may be NULL).
 *  - All arithmetic is unsigned integer, modulo 2^64.  All data is little-endian.
 *  - All structs below are plain data with natural alignment and no padding.
 */
#ifndef FDY_H
#define FDY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FDY_VERSION 300 /* major*10000 + minor*100 + patch */

/* ---- return codes ------------------------------------------------------------------ */
#define FDY_OK 0
#define FDY_ERR_INVALID_ARG (-1) /* null/misaligned pointer, size out of range        */
#define FDY_ERR_TABLE (-2)       /* allocation table not sorted / overlapping / empty */
#define FDY_ERR_CAPACITY (-3)    /* reserved: reported through FDY_ST_CAPACITY         */
#define FDY_ERR_HIP (-4)         /* a HIP call or kernel launch failed                */
#define FDY_ERR_WORKSPACE (-5)   /* workspace pointer null, misaligned or too small   */
#define FDY_ERR_ORDER (-6)       /* a host list is not strictly ascending by location */
#define FDY_ERR_IO (-7)          /* fdy_archive.h: a file could not be opened, mapped, written */
#define FDY_ERR_FORMAT (-8)      /* fdy_archive.h: not an archive, or a damaged container       */
#define FDY_ERR_CHECKSUM (-9)    /* fdy_archive.h: a stored sum does not match the bytes        */
#define FDY_ERR_CONTENT (-10)    /* fdy_archive.h: the sections contradict each other           */

/* ---- device status bits (OR-ed into *d_status) ------------------------------------- */
#define FDY_ST_CAPACITY 0x1u  /* scan: more hits than reloc_capacity; *d_count = needed
                                 (derive: more entries than ovr_capacity)               */
#define FDY_ST_BAD_INDEX 0x2u /* an entry's word/region/node/template index was out of
                                 range and the entry was skipped                        */
#define FDY_ST_BAD_SIZE 0x4u  /* materialize: out_words_per_map / out_nodes_total do not
                                 equal the sums the device computed; nothing written
                                 (derive: a graph and its template differ in length)     */
#define FDY_ST_SPIN 0x8u      /* scan: a bounded wait on a predecessor tile ran out      */
#define FDY_ST_BAD_ORDER 0x10u /* materialize: a relocation, override, grid-override or
                                 patch list is not strictly ascending by location; the
                                 output is unspecified (entries may be missing)          */

#define FDY_ST_BAD_PREPARED 0x20u /* scan: d_prepared was not made by fdy_scan_table_prepare
                                    for this table and at least this many words; nothing
                                    was read from it and no output was written            */

/* ---- plain-data records ------------------------------------------------------------ */

/* One allocation of the deterministic layout: the half-open byte range [base, base+size).
 * A table is sorted by strictly ascending base, has size >= 1, base+size does not wrap
 * and ranges do not overlap (they may touch).  Section 4.1.1 / Section 5.1: allocations
 * are placed one after another from a fixed base, so the record of them is such a table. */
typedef struct {
  uint64_t base;
  uint64_t size;
} fdy_alloc; /* 16 B */

/* One kernel node of a captured graph, reduced to the fields the fingerprint and the
 * launch-dimension output use (Appendix B lists the full record).  kernel_id stands for
 * the (binary content hash, function name) key of Section 4.1.2.  flags carries the node
 * type / kernel-node attributes that Section 5.3 counts as topology (bit 0: communication
 * node). blob_len is the byte length of the node's argument buffer, a multiple of 8. */
typedef struct {
  uint64_t kernel_id;
  uint32_t grid[3];
  uint32_t block[3];
  uint32_t blob_len;
  uint32_t flags;
} fdy_node; /* 40 B */

/* One relocation: 8-byte word number `word` of the scanned array holds a pointer into
 * allocation `region`, `offset` bytes above its base. */
typedef struct {
  uint32_t word;
  uint32_t region;
  uint64_t offset;
} fdy_reloc; /* 16 B */

/* Per-graph scalar override: store the 32-bit `value` at byte offset `byte_off`
 * (a multiple of 4) of the graph's argument blob.  Section 3: graphs of one topology
 * differ only in per-node parameters such as a batch-size argument. */
typedef struct {
  uint32_t byte_off;
  uint32_t value;
} fdy_ovr32; /* 8 B */

/* Per-graph launch-dimension override: node `node` of the graph gets grid dims `grid`. */
typedef struct {
  uint32_t node;
  uint32_t grid[3];
} fdy_grid_ovr; /* 16 B */

/* Rank-dependent 64-bit patch: 8-byte word `word` (relative to the template's first word)
 * is replaced by `value` (communication handle, {rank,nranks}, peer-buffer address).
 * Section 4.2.2: LOAD substitutes the real handle and updates rank-specific arguments. */
typedef struct {
  uint32_t word;
  uint32_t reserved; /* must be 0 */
  uint64_t value;
} fdy_patch; /* 16 B */

/* ---- fingerprint field mask -------------------------------------------------------- */
#define FDY_FP_KERNEL_ID 0x01u
#define FDY_FP_GRID_X 0x02u
#define FDY_FP_GRID_Y 0x04u
#define FDY_FP_GRID_Z 0x08u
#define FDY_FP_BLOCK 0x10u
#define FDY_FP_BLOB_LEN 0x20u
#define FDY_FP_FLAGS 0x40u
#define FDY_FP_ALL 0x7fu

/* ---- library ----------------------------------------------------------------------- */

/* FDY_VERSION of the built library. */
int fdy_version(void);

/* Static, NUL-terminated description of a return code (never NULL). */
const char* fdy_strerror(int code);

/* Host-side check of an allocation table held in HOST memory against the rules stated at
 * fdy_alloc.  Returns FDY_OK, FDY_ERR_INVALID_ARG (null pointer with n_alloc > 0) or
 * FDY_ERR_TABLE; on FDY_ERR_TABLE *h_bad_index (may be NULL) is the first offending entry.
 * An empty table (n_alloc == 0) is valid: nothing is a pointer. */
int fdy_table_validate(const fdy_alloc* h_table, uint32_t n_alloc, uint32_t* h_bad_index);

/* Inverse of a base map (host).  A base map places region r of `h_table` at h_new_base[r];
 * the relaxation of Section 4.1.1 works in both directions: blobs that hold pointers into
 * the NEW layout are taken back to the captured one (or classified against the new layout)
 * by running the same scan with the new layout as its table.  This call builds that table:
 *   h_inv_table[k]  = {h_new_base[r_k], size of region r_k}, ascending by new base
 *   h_inv_base[k]   = captured base of region r_k      (the base map of the way back)
 *   h_inv_region[k] = r_k                               (may be NULL)
 * so that fdy_scan_rebase(words, h_inv_table, h_inv_base) undoes
 * fdy_scan_rebase(words, h_table, h_new_base) on every pointer, and fdy_scan_pointers over
 * h_inv_table reports region k for captured region r_k.  All arrays are HOST memory of
 * n_alloc entries, outputs distinct from inputs.  FDY_ERR_INVALID_ARG: a null pointer with
 * n_alloc > 0; FDY_ERR_TABLE: h_table is not valid, or the regions overlap or wrap in the new
 * layout (then the way back is not a function; outputs are unspecified). */
int fdy_layout_invert(const fdy_alloc* h_table, const uint64_t* h_new_base, uint32_t n_alloc,
                      fdy_alloc* h_inv_table, uint64_t* h_inv_base, uint32_t* h_inv_region);

/* ---- capture-window replay: a recorded layout placed in a new address range ----------
 * Section 4.1.1 ("capture-window" allocations recorded at SAVE are issued again at LOAD, so
 * that every address the graphs expect exists) and Section 5.1: the deterministic layout
 * keeps every allocation at the same distance from the start of its address range, whatever
 * that start is.  Given the table that a recording run left (h_recorded[n], in an address
 * range that started at recorded_start), this places each allocation at the same distance
 * from new_start in a range of new_capacity bytes whose first new_used bytes are already
 * taken, and writes h_new_base[i] = new_start + (h_recorded[i].base - recorded_start): the
 * base map of the recorded table that fdy_materialize and fdy_scan_rebase take.  Host call,
 * host pointers.
 *   FDY_ERR_INVALID_ARG  n > 0 and a null pointer
 *   FDY_ERR_TABLE        h_recorded is not a valid table, or starts below recorded_start
 *   FDY_ERR_ORDER        the first allocation would start inside the first new_used bytes
 *   FDY_ERR_CAPACITY     the last allocation would end behind new_capacity bytes, or behind
 *                        the end of the address space
 * On any error h_new_base is not written. */
int fdy_layout_replay(const fdy_alloc* h_recorded, uint32_t n, uint64_t recorded_start, uint64_t new_start,
                      uint64_t new_capacity, uint64_t new_used, uint64_t* h_new_base);

/* ---- (a1) pointer scan -------------------------------------------------------------
 * Classifies every 8-byte word of d_words against the allocation table and emits the
 * relocation table (Section 4.1.1 and Section 2.2 give the need; the paper itself avoids
 * the scan by forcing an identical layout).  For word j with value w, let i be the last
 * table entry with base[i] <= w; j is a hit iff such i exists and w - base[i] < size[i].
 * Hits are written to d_relocs in ascending j as {word=j, region=i, offset=w-base[i]}.
 *
 *   d_words          [n_words] device, 16-byte aligned; n_words <= 2^32 - 256
 *   d_table          [n_alloc] device, 16-byte aligned, valid per fdy_table_validate
 *                    (the caller validates; an invalid table gives unspecified relocation
 *                    contents but no out-of-bounds access)
 *   d_relocs         [reloc_capacity] device, 16-byte aligned
 *   d_count          device uint64_t: total number of hits, also when it exceeds
 *                    reloc_capacity (then only the first reloc_capacity entries are
 *                    written and FDY_ST_CAPACITY is raised)
 *   d_workspace      device, 256-byte aligned, at least fdy_scan_workspace_bytes() bytes;
 *                    contents on entry are irrelevant, contents on exit are unspecified.
 *                    The size is the search hierarchy built from the table (about 30 bytes
 *                    per allocation beyond 16,384 of them: packed copies of the table, and
 *                    room for one new base per allocation beside them, which
 *                    fdy_scan_pointers_rebase fills per call) and 8 bytes per 4,096 words;
 *                    0 is returned for n_words beyond the limit above.
 *                    Optional staging area: where more than 3 words in 8 lie inside the
 *                    table's span (word-dense inputs), the hits of such a stretch are either
 *                    staged (a workspace of fdy_scan_workspace_bytes() +
 *                    fdy_scan_staging_bytes() bytes or more: up to 160 MiB, independent of
 *                    the table) or found by searching the stretch a second time (any smaller
 *                    workspace; about 1.6 times slower on inputs that are dense throughout).
 *                    Same results either way
 *   d_prepared       NULL, or the table's prepared form (see fdy_scan_table_prepare below)
 *   d_status         device uint32_t or NULL
 */
size_t fdy_scan_workspace_bytes(uint64_t n_words, uint32_t n_alloc);
size_t fdy_scan_staging_bytes(uint64_t n_words);
int fdy_scan_pointers(const uint64_t* d_words, uint64_t n_words, const fdy_alloc* d_table,
                      uint32_t n_alloc, fdy_reloc* d_relocs, uint64_t reloc_capacity,
                      uint64_t* d_count, const void* d_prepared, void* d_workspace,
                      size_t workspace_bytes, uint32_t* d_status, void* hip_stream);

/* ---- prepared table (optional; one per allocation table) ------------------------------
 * The layout, hence the allocation table, is fixed for the life of an archive (Section
 * 4.1.1), while blobs are scanned many times against it.  What a scan derives from the table
 * alone (its search hierarchy) can therefore be built once, into a device buffer that the
 * caller owns, and handed to every scan of that table as d_prepared; such a call launches
 * one kernel where it otherwise launches two.  The buffer also holds the scan's counters
 * (work ticket, per-chunk totals), which a scan leaves zeroed behind it:
 *   - calls that share a prepared table must not overlap in time (one stream, or ordered by
 *     events); read-only sharing is not possible;
 *   - after a call that returned FDY_ERR_HIP, or that raised FDY_ST_SPIN, prepare it again;
 *   - the buffer belongs to the table at d_table (same address and contents), to n_words <=
 *     max_words and to the process's tuning at the time; the device checks this and raises
 *     FDY_ST_BAD_PREPARED, writing nothing, when it does not hold.
 * With d_prepared the workspace only holds the optional staging area of dense inputs
 * (fdy_scan_staging_bytes; NULL or anything smaller: none).  d_prepared == NULL: the call
 * builds the hierarchy into its workspace itself.
 *
 *   fdy_scan_table_bytes    size of the buffer for a table of n_alloc entries that serves
 *                           scans of up to max_words words (0: max_words out of range)
 *   fdy_scan_table_prepare  enqueues the build; d_prepared device, 256-byte aligned
 */
size_t fdy_scan_table_bytes(uint32_t n_alloc, uint64_t max_words);
int fdy_scan_table_prepare(const fdy_alloc* d_table, uint32_t n_alloc, uint64_t max_words,
                           void* d_prepared, size_t prepared_bytes, void* hip_stream);

/* ---- fused scan + rebase (variant; a1 + c1 + c2 in one pass) ------------------------
 * For one new layout and no templating (a new instance whose addresses differ, Section
 * 4.1.1 relaxed; argument buffers are opaque, Section 2.2), the relocation table need not
 * exist: with i, offset as in fdy_scan_pointers,
 *   d_out_words[j] = d_new_base[i] + offset (mod 2^64)   if word j is a hit,
 *   d_out_words[j] = d_words[j]                          otherwise,
 * which equals fdy_scan_pointers followed by fdy_materialize with one source graph, one
 * base map and no overrides or patches.  Every input word is read once and every output
 * word written once.
 *
 *   d_words, d_table as for fdy_scan_pointers
 *   d_new_base       [n_alloc] device, 8-byte aligned
 *   d_out_words      [n_words] device, 16-byte aligned; either d_words itself (in place) or
 *                    an array that does not overlap it (anything else: FDY_ERR_INVALID_ARG)
 *   d_count          device uint64_t: number of hits
 *   d_prepared, d_workspace   as for fdy_scan_pointers (same size query)
 *   d_status         device uint32_t or NULL
 */
int fdy_scan_rebase(const uint64_t* d_words, uint64_t n_words, const fdy_alloc* d_table,
                    uint32_t n_alloc, const uint64_t* d_new_base, uint64_t* d_out_words,
                    uint64_t* d_count, const void* d_prepared, void* d_workspace,
                    size_t workspace_bytes, uint32_t* d_status, void* hip_stream);

/* ---- scan with rebased output (a1 + c1 + c2 for one layout, relocation table kept) ------
 * fdy_scan_pointers and fdy_scan_rebase in one pass over the words: the relocation table is
 * written exactly as by fdy_scan_pointers (ascending, same d_count / capacity / status rules)
 * AND d_out_words receives what fdy_scan_rebase would write.  This is the whole of (c) for an
 * archive whose graphs are their own templates and that is instantiated for one new layout
 * (the inter-rank sense of a template, Section 4.2.2: every rank takes the same captured
 * blobs): the words are read once instead of once by the scan and once by the
 * materialization, while the table stays available for further base maps (fdy_materialize)
 * and for storing with the archive.  Overrides and rank patches are not applied by this call.
 *
 *   d_words, d_table, d_relocs, reloc_capacity, d_count, d_prepared, d_workspace, d_status
 *                    as for fdy_scan_pointers (same size query)
 *   d_new_base       [n_alloc] device, 8-byte aligned
 *   d_out_words      [n_words] device, 16-byte aligned, must not overlap d_words
 *                    (FDY_ERR_INVALID_ARG; in place is what fdy_scan_rebase offers)
 * A hit beyond reloc_capacity is still rebased in d_out_words. */
int fdy_scan_pointers_rebase(const uint64_t* d_words, uint64_t n_words, const fdy_alloc* d_table,
                             uint32_t n_alloc, fdy_reloc* d_relocs, uint64_t reloc_capacity,
                             uint64_t* d_count, const uint64_t* d_new_base, uint64_t* d_out_words,
                             const void* d_prepared, void* d_workspace, size_t workspace_bytes,
                             uint32_t* d_status, void* hip_stream);

/* Variant of fdy_scan_pointers for pointers at 4-byte alignment (argument buffers are opaque
 * byte strings, Section 2.2 / Appendix B: a packed structure may hold a pointer at any
 * 4-byte offset).  The array is read as n_units 32-bit little-endian units; position q
 * (0 <= q < n_units - 1) stands for the 64-bit value whose low half is unit q and whose high
 * half is unit q + 1, and every position is classified like a word of fdy_scan_pointers.
 * Relocations come out ascending by position, reloc.word = q (so an 8-byte-aligned pointer
 * at word j appears as q = 2 j, and the call finds a superset of what fdy_scan_pointers finds
 * on the same bytes).  d_units must be 16-byte aligned; n_units - 1 <= 2^32 - 257; the
 * workspace is sized by fdy_scan_workspace_bytes(n_units, n_alloc).  Arguments, errors and
 * status bits otherwise as for fdy_scan_pointers.  Reads the array once (each unit serves
 * two positions) and writes the relocation table once. */
int fdy_scan_pointers_stride4(const uint32_t* d_units, uint64_t n_units, const fdy_alloc* d_table,
                              uint32_t n_alloc, fdy_reloc* d_relocs, uint64_t reloc_capacity,
                              uint64_t* d_count, const void* d_prepared, void* d_workspace,
                              size_t workspace_bytes, uint32_t* d_status, void* hip_stream);

/* ---- (a2) relocation segmentation ---------------------------------------------------
 * For each boundary d_word_off[s], s in [0, n_off): d_reloc_off[s] = number of entries of
 * d_relocs[0, min(*d_count, reloc_capacity)) whose word is < d_word_off[s] (lower bound in
 * the ascending table).  With d_word_off = the archive's per-graph word offsets [G+1] this
 * yields each graph's slice of the relocation table. */
int fdy_reloc_segment(const fdy_reloc* d_relocs, const uint64_t* d_count,
                      uint64_t reloc_capacity, const uint64_t* d_word_off, uint32_t n_off,
                      uint64_t* d_reloc_off, void* hip_stream);

/* ---- (b) topology fingerprint -------------------------------------------------------
 * Section 4.2.1 / Section 5.3: a key per graph over its structural properties; graphs
 * with equal keys form one group served by one template.  The paper leaves the key
 * function open; this library fixes it as follows (all mod 2^64):
 *   mix(x): x ^= x>>30; x *= 0xbf58476d1ce4e5b9; x ^= x>>27; x *= 0x94d049bb133111eb;
 *           x ^= x>>31                      (the SplitMix64 output function)
 *   P = 0x9e3779b97f4a7c15
 *   node_hash(n): fields not selected by field_mask read as 0 (FDY_FP_BLOCK selects all
 *           three block dims), then
 *           a = mix(kernel_id + P);            a = mix(a ^ (grid[0]  | grid[1]  << 32));
 *           a = mix(a ^ (grid[2] | block[0] << 32)); a = mix(a ^ (block[1] | block[2] << 32));
 *           a = mix(a ^ (blob_len | flags << 32))
 *   key(g): H = mix(N_g); for each node in order: H = H*P + node_hash(node); key = mix(H)
 *   template_id[g]: dense id, in order of first appearance, of g's key
 *   tmpl_graph[t]: the first graph (lowest index) whose template_id is t
 *
 *   d_nodes          device, 8-byte aligned; graph g owns nodes [d_node_off[g], d_node_off[g+1])
 *   d_node_off       [n_graphs+1] device, non-decreasing
 *   d_keys           [n_graphs] out
 *   d_template_id    [n_graphs] out
 *   d_tmpl_graph     [n_graphs] out (first *d_n_templates entries meaningful) or NULL
 *   d_n_templates    device uint32_t out
 *   n_graphs         <= 2^20
 *   d_workspace      device, 256-byte aligned, >= fdy_fingerprint_workspace_bytes(n_graphs)
 *                    bytes; only archives of more than 8,192 graphs use it (NULL is accepted
 *                    up to there); contents on entry are irrelevant
 * Grouping takes time linear in the number of graphs (a hash table over the keys).
 */
size_t fdy_fingerprint_workspace_bytes(uint32_t n_graphs);
int fdy_fingerprint(const fdy_node* d_nodes, const uint64_t* d_node_off, uint32_t n_graphs,
                    uint32_t field_mask, uint64_t* d_keys, uint32_t* d_template_id,
                    uint32_t* d_tmpl_graph, uint32_t* d_n_templates, void* d_workspace,
                    size_t workspace_bytes, void* hip_stream);

/* (a2) and (b) in one launch: fdy_reloc_segment over the archive's per-graph word offsets
 * (d_word_off and d_reloc_off are [n_graphs + 1]) and fdy_fingerprint, same results.  The
 * archives of Section 6.1 (one graph per batch size of a 36- or 94-layer model) are so small
 * that a LOAD step is bound by the number of launches, not by bandwidth.  With a prepared
 * table (any buffer made by fdy_scan_table_prepare; its first block holds a counter that this
 * call finds zero and leaves zero, so calls sharing it must not overlap) and at most 8,192
 * graphs the grouping runs in the same launch, in the last block to finish; with d_prepared
 * NULL it is a launch of its own.  Other arguments as for the two plain calls. */
int fdy_segment_fingerprint(const fdy_reloc* d_relocs, const uint64_t* d_count, uint64_t reloc_capacity,
                            const uint64_t* d_word_off, uint64_t* d_reloc_off,
                            const fdy_node* d_nodes, const uint64_t* d_node_off, uint32_t n_graphs,
                            uint32_t field_mask, uint64_t* d_keys, uint32_t* d_template_id,
                            uint32_t* d_tmpl_graph, uint32_t* d_n_templates, void* d_prepared,
                            void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* ---- override derivation (SAVE side of templating; variant, after (b)) ----------------
 * Within a topology group the graphs differ only in per-node parameters (Section 4.2.1,
 * Section 5.3), so a non-template graph is stored as what differs from its template.  For
 * graph g let s = d_tmpl_graph[d_graph_tmpl[g]] (as fdy_fingerprint produces them); for every
 * byte offset b, a multiple of 4, at which the 32-bit little-endian value of g's blob
 * differs from s's, the entry {byte_off = b, value = g's value} is written; ascending b per
 * graph, graphs in order.  d_ovr_off[g] = entries before graph g, d_ovr_off[n_graphs] = the
 * total, also when it exceeds ovr_capacity (then only the first ovr_capacity entries are
 * written and FDY_ST_CAPACITY is raised).  The lists are what fdy_materialize takes as ovr /
 * ovr_off when the same array of words is its source archive: template + overrides = graph.
 * A word that holds a pointer and differs from the template's is reported like any other;
 * such a graph does not share its template's parameters and should not share its group.
 *
 *   d_words          device, 8-byte aligned: all graphs' words; graph g owns words
 *                    [d_word_off[g], d_word_off[g+1])
 *   n_words_total    host copy of d_word_off[n_graphs] (sizes the workspace; a mismatch
 *                    raises FDY_ST_BAD_SIZE and yields no entries)
 *   d_graph_tmpl     [n_graphs] template id of each graph
 *   d_tmpl_graph     [n_templates] source graph of each template
 *   d_ovr            [ovr_capacity] out, 8-byte aligned
 *   d_ovr_off        [n_graphs+1] out
 *   d_workspace      device, 256-byte aligned, >= fdy_derive_workspace_bytes() bytes
 *   d_status         device uint32_t or NULL: FDY_ST_BAD_INDEX for a template id or source
 *                    graph out of range, FDY_ST_BAD_SIZE for a graph whose word count
 *                    differs from its template's (such graphs get no entries)
 *   n_graphs <= 2^20, n_words_total < 2^40, every graph below 2^29 words (32-bit offsets)
 */
size_t fdy_derive_workspace_bytes(uint64_t n_words_total, uint32_t n_graphs);
int fdy_derive_overrides(const uint64_t* d_words, uint64_t n_words_total, const uint64_t* d_word_off,
                         uint32_t n_graphs, const uint32_t* d_graph_tmpl,
                         const uint32_t* d_tmpl_graph, uint32_t n_templates, fdy_ovr32* d_ovr,
                         uint64_t ovr_capacity, uint64_t* d_ovr_off, void* d_workspace,
                         size_t workspace_bytes, uint32_t* d_status, void* hip_stream);

/* ---- (c) template materialization ---------------------------------------------------
 * For every base map m and every output graph g (Section 4.2.1: prepare the parameter
 * sets of the non-template graphs; Section 4.2.2: patch rank-dependent state), in this
 * stage order, a later stage overwriting an earlier one at the same location:
 *   c1  out[m][g]        = copy of the argument blob of template t = graph_tmpl[g]
 *   c2  out[m][g][k]     = new_base[m][region] + offset   for each reloc of the template,
 *                          k = reloc.word - (first word of the template)
 *   c3  store32(out[m][g] bytes, byte_off, value)          for each override of graph g
 *   c4  out[m][g][word]  = value   for each patch of (t, map_rank[m]), if map_rank != NULL
 * and, once per graph (launch dims do not depend on the map):
 *   dims[g][n] = {grid xyz, block xyz} of the template's node n, then grid replaced for
 *                each grid override of graph g.
 *
 * The template of id t is source graph s = tmpl_graph[t] of the "source archive": words
 * [src_word_off[s], src_word_off[s+1]) of src_words, nodes [src_node_off[s], ..[s+1]) of
 * src_nodes, relocs [src_reloc_off[s], ..[s+1]) of relocs with reloc.word indexing
 * src_words (exactly what fdy_scan_pointers + fdy_reloc_segment produce for the archive).
 * Each reloc / override / grid-override / patch list is strictly ascending by location (the
 * slices of a list that fall into an output tile are found by binary search).  The device
 * verifies it for every list it reads: a list out of order, or with a location twice, raises
 * FDY_ST_BAD_ORDER and leaves the output unspecified, without any out-of-bounds access.  The
 * lists of a template that no output graph uses are not read.
 *
 * Output layout: d_out_words is [n_maps][out_words_per_map], map-major; inside a map the
 * graphs follow in order g = 0..n_graphs-1, each with the word count of its template.
 * d_out_dims is [out_nodes_total][6] uint32 (grid xyz, block xyz), graphs in order, or
 * NULL to skip the dims output.
 */
typedef struct {
  /* host scalars */
  uint32_t n_src_graphs; /* S: graphs in the source archive arrays                   */
  uint32_t n_templates;  /* T                                                          */
  uint32_t n_graphs;     /* G: output graphs per map                                   */
  uint32_t n_maps;       /* M                                                          */
  uint32_t n_alloc;      /* A: regions per base map                                    */
  uint32_t n_ranks;      /* R: rank patch tables per template (0 when map_rank==NULL)  */
  uint64_t out_words_per_map; /* sum over g of words(template(g))                      */
  uint64_t out_nodes_total;   /* sum over g of nodes(template(g)); 0 if d_out_dims NULL */
  /* device arrays */
  const uint64_t* src_words;     /* 16-byte aligned                                    */
  const uint64_t* src_word_off;  /* [S+1]                                              */
  const fdy_node* src_nodes;     /* may be NULL when d_out_dims is NULL                */
  const uint64_t* src_node_off;  /* [S+1]                                              */
  const fdy_reloc* relocs;       /* 16-byte aligned                                    */
  const uint64_t* src_reloc_off; /* [S+1]                                              */
  const uint32_t* tmpl_graph;    /* [T] source graph of each template                  */
  const uint32_t* graph_tmpl;    /* [G] template of each output graph                  */
  const fdy_ovr32* ovr;          /* overrides, all graphs concatenated                 */
  const uint64_t* ovr_off;       /* [G+1]                                              */
  const fdy_grid_ovr* govr;      /* grid overrides, all graphs concatenated            */
  const uint64_t* govr_off;      /* [G+1]                                              */
  const uint64_t* new_base;      /* [M][A] row-major                                   */
  const uint32_t* map_rank;      /* [M] rank of each map, or NULL: no patches          */
  const fdy_patch* patch;        /* patches, index t*R+r concatenated                  */
  const uint64_t* patch_off;     /* [T*R+1]                                            */
} fdy_mat_desc;

/* Workspace size for fdy_materialize with this descriptor (only the host scalars are
 * read).  0 is returned for a descriptor whose scalars are out of range. */
size_t fdy_materialize_workspace_bytes(const fdy_mat_desc* h_desc);

/*   h_desc       HOST struct; read during the call only
 *   d_out_words  device, 16-byte aligned, n_maps*out_words_per_map words
 *   d_out_dims   device, 8-byte aligned, out_nodes_total*6 uint32, or NULL
 *   d_workspace  device, 256-byte aligned, >= fdy_materialize_workspace_bytes(h_desc)
 *   d_status     device uint32_t or NULL
 * Limits: n_graphs, n_src_graphs, n_templates <= 2^20; n_maps <= 65535; every template
 * < 2^32 words; out_words_per_map < 2^40. */
int fdy_materialize(const fdy_mat_desc* h_desc, uint64_t* d_out_words, uint32_t* d_out_dims,
                    void* d_workspace, size_t workspace_bytes, uint32_t* d_status,
                    void* hip_stream);

/* ---- fdy_materialize without a workspace ----------------------------------------------
 * For callers that cannot allocate device memory where they call from: code that runs under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation,
 * same outputs and status bits as fdy_materialize; the tile table and the other per-call
 * tables lie in a fixed array of fdy_materialize_static_limit() bytes (4 MiB) inside the
 * loaded library, one copy per GPU, held until the process ends.  The call allocates and
 * frees nothing.
 *   - FDY_ERR_WORKSPACE: the descriptor needs more than the fixed array holds
 *     (fdy_materialize_workspace_bytes(h_desc) > fdy_materialize_static_limit()); use
 *     fdy_materialize then.
 *   - Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU
 *     (different streams, no ordering between them) race.  Calls on one stream are fine.
 *   - The first call on each device looks the array's address up (with that device current);
 *     make it outside graph capture. */
size_t fdy_materialize_static_limit(void);
int fdy_materialize_static(const fdy_mat_desc* h_desc, uint64_t* d_out_words, uint32_t* d_out_dims,
                           uint32_t* d_status, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FDY_H */
