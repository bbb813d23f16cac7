// fdy_scan.hip - (a1) pointer scan and (a2) relocation segmentation for gfx950.
//
// The scan classifies every 8-byte word of the captured argument blobs against the sorted
// allocation table (the relaxation of Section 4.1.1's identical-layout requirement: find
// every embedded pointer kernel-agnostically, because argument buffers are opaque -
// Section 2.2, Appendix B).  It is one streaming pass over the words.  What bounds it, in
// this order, as measured on MI355X: (1) the dependent round trips of a search (LDS, then L2,
// then the memory side), which a wave pays once per batch of candidates and which only other
// waves and other batches can hide; (2) what the candidates pull through the memory fabric
// once the table outgrows the 4 MiB L2 of an XCD (a 128-byte table line per candidate is
// 2.5x the bytes of the words themselves at 15 % candidates); (3) HBM bandwidth for the words.
// Hence: candidates of several sub-tiles are searched together in dense rounds, every level
// of the hierarchy is fetched as one whole node, and large tables are read through a packed
// copy of half the size.
//
// Work decomposition.  A persistent workgroup of 8 waves stages the top level of the table
// hierarchy in LDS once.  Work is handed out by an atomic ticket, but not per sub-tile
// (same-address atomics complete at under 1e8/s on this chip, which alone would cap a
// 1 GiB scan near 1.3 TB/s): a workgroup draws a chunk of 32 sub-tiles (512 words each)
// per ticket: two groups, in each of which every wave owns two consecutive sub-tiles,
// sub-tile = base + (group*8 + wave)*2 + row.  Tickets are drawn two rounds ahead, so the
// words of the next group (of this chunk or the next) are already in flight while a group is
// searched.  Per group a wave
//   1. takes its 2 x 8 words per lane (16-byte coalesced non-temporal loads) and rejects
//      every word outside the table's span with one subtract-and-compare;
//   2. compacts the surviving candidates of both sub-tiles, in word order, into its private
//      LDS queue (wave ballot + popcount ranks), so that the interval search runs on dense
//      rounds of 64 lanes and its round trips are paid once per group, not per sub-tile;
//   3. searches the hierarchy, up to three rounds (three candidates per lane) interleaved so
//      that their dependent steps overlap:
//        level 0  sampled bases (every S-th, S = 8^k) as 31-bit keys (base - span_lo) >> sh
//                 in LDS, behind a bucket index over the key space (which keys can the
//                 answer be among), so that a search reads 3-5 keys, not 14; a key equal to
//                 the candidate's is ambiguous and is settled against the exact base in the
//                 table (rare);
//        level j  k-1 packed arrays "every 8^j-th base" in global memory, small enough to
//                 stay in L2: one 64-byte node of 8 keys per level, fetched whole;
//        leaf     8 consecutive {base,size} entries: from the packed copy of the table (64
//                 bytes per line) when the table is large, else from the table itself;
//        level 1 and the leaf are read through 32-byte copies (two loads per candidate and
//        level instead of four, and half the footprint in L2) where the table's nodes and
//        lines mostly fit them, which layouts made of whole mapping granules do;
//      region and offset of each candidate stay in registers, its word index in LDS;
//   4. counts its hits into LDS.
// One workgroup barrier per chunk makes the counts and the next ticket visible.  The output
// position of the chunk comes from a decoupled look-back over per-CHUNK state words (flag and
// value packed in one 64-bit word, agent-scope relaxed atomics), walked by one wave per
// workgroup: a few hundred chunks are in flight at any time, so the walk is a handful of
// 64-wide steps (a look-back over per-sub-tile states would walk thousands of entries).
// The look-back runs one round late: a chunk's results wait in registers while the next
// chunk is searched, and by then the chunks before it have published their totals, so no
// workgroup stalls on another one.  The waves then write their relocation entries from
// registers in ascending word order.
// The input is read exactly once and the relocation table written exactly once.
//
// A group with more than 384 candidates (over a third of its words inside the table's span:
// more than the registers keep results for) is handled sub-tile by sub-tile in windows of
// queue size, one round at a time; its hits go to a staging area in the workspace as complete
// entries (each wave has room for one entry per word of the two chunks it has in flight) and
// are copied to their place when the chunk's position is known.  Slower per candidate than
// the register path (single rounds, and the entries travel twice), same result.
//
// Variant at 4-byte stride (fdy_scan_pointers_stride4): the same kernel with kHalf set reads
// the array as 32-bit units and treats every unit index as a position whose value is that
// unit and the next one; only the loader and the numbering of positions differ.
//
// Variant with a rebased output (fdy_scan_pointers_rebase; kOut): the same ordered scan also
// writes every word, hits rebased, to a second array, so that an archive whose graphs are
// their own templates needs no second pass over the words (Section 4.2.2: every rank takes the
// same captured blobs and differs only in its layout).  A wave keeps the sub-tiles of its
// group in LDS as loaded, queues only the candidates' positions, writes new_base[region] +
// offset over each hit's copy and streams the copy out with the 16-byte stores a copy would
// use (scattered 8-byte fix-ups into lines that have left L2 cost a third more time).  The
// LDS for the copies comes from the level-0 keys, which this variant keeps as 16-bit
// distances inside their bucket.  A small launch ahead of the scan lays each compact table line
// and the new bases of its eight regions side by side in one 128-byte record, so that a hit's
// new base is a second request to the line the search has just fetched.
//
// The table's part of all this (hierarchy, packed copies) depends on the table alone and can
// be built once per archive (fdy_scan_table_prepare); the per-call state (ticket, chunk
// states, counters) then lives in the same buffer and is zeroed again by the last workgroup
// to finish, so that a scan is one launch.
//
// Tickets are handed out in increasing order and a wave only ever waits for chunks with
// smaller numbers, which are already owned by resident workgroups; the wait is bounded by a
// spin limit after which FDY_ST_SPIN is raised and the kernel still terminates.
//
// Loops whose bodies hold a whole search are not written as loops: past a size the optimizer
// declines to unroll even a `#pragma unroll` loop, and a rolled loop indexes the
// register-resident results dynamically, which sends them to scratch memory.  Groups are
// therefore instantiated one by one from a generic lambda with a compile-time index.
#include <type_traits>

#include "fdy_device.hpp"
#include "fdy_internal.h"

namespace fdy {
namespace {

constexpr u64 kMaxWords = (1ull << 32) - 256;  // word and reloc indices are 32-bit
constexpr int kWaves = 8;                      // waves per workgroup
constexpr int kBlock = kWaves * 64;
constexpr int kLoads = 4;                      // 16-byte loads per lane per sub-tile
constexpr int kWpl = 2 * kLoads;               // words per lane per sub-tile
constexpr int kSub = 64 * kWpl;                // words per sub-tile (512)
constexpr int kGroupsBig = 2, kGBig = 2;       // large inputs: a wave takes 2 groups of 2 sub-tiles per ticket
constexpr int kGroupsSmall = 1, kGSmall = 1;   // small inputs: more, smaller chunks fill the chip
constexpr int kQcap = 192;                     // queue entries per wave
constexpr int kRegRounds = 3;                  // rounds of 64 candidates per sub-tile kept in registers
constexpr int kMaxMid = 6;                     // packed levels in global memory
constexpr u32 kMiss = 0xffffffffu;
constexpr u32 kStageWgs = 320;                 // most workgroups the scan launches (staging is sized for them)

struct ScanParams {
  const u64* words;
  u64 n_words;
  const fdy_alloc* table;
  u32 n_alloc;
  fdy_reloc* relocs;
  u64 capacity;
  u64* d_count;
  u32* ticket;
  const u32* top;  // [top_n] level-0 keys, padded with 0xffffffff
  const unsigned short* bstart;  // [n_buckets + 1] level-0 keys below each bucket's first key value
  u32 bucket_log2;  // log2(n_buckets)
  const u64* mid[kMaxMid];  // mid[j-1] = every 8^j-th base, padded with ~0
  const uint4* leaf;        // packed table, 64 bytes per 8 entries (null: not built)
  const uint4* cmid;        // compact copy of packed level 1, 32 bytes per node of 8 keys (null: not built)
  const uint4* cleaf;       // compact copy of the table, 32 bytes per 8 entries (null: not built)
  const uint4* leafmap;     // ordered scan with output: 128 bytes per 8 entries, the compact line and
                            // behind it the eight regions' new bases (null: not built)
  u64* cstate;     // [n_chunks] per-chunk totals / inclusive prefixes
  u32* done;       // workgroups that have finished (the last one resets the state behind it)
  u64* acc;        // fused scan + rebase: hits so far
  u32 n_chunks;
  u32 self_clean;  // the state (ticket, chunk states, counters) is left zeroed for the next call
  const u64* prepared;  // the caller's prepared table (its header is checked on the device), or null
  u32 top_log2;         // the tuning that the hierarchy's layout depends on
  fdy_reloc* stage;  // [grid][2][sub-tiles of a chunk * kSub]: staged entries of dense groups; null:
                     // no staging area, dense groups are searched twice
  u32 n_sub;       // sub-tiles
  u32 top_n;       // power of two
  u32 levels;      // k: 8-ary levels below level 0, the table line included
  u32 f0_log2;     // level 0 samples every (2^f0_log2 * 8^k)-th base
  u32* d_status;
  u32 spin_limit;
  const u64* new_base;  // with a rebased output only: [n_alloc]
  u64* out;             // with a rebased output only: [n_words]
  u32 key_bits;         // width of the level-0 keys: 31 (32-bit keys in LDS) or 16 + bucket_log2 (16-bit keys)
};

constexpr u64 kFlagAgg = 1ull << 62;
constexpr u64 kFlagInc = 2ull << 62;
constexpr u64 kValMask = (1ull << 62) - 1;

__device__ __forceinline__ u64 ld_state(const u64* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_state(u64* p, u64 v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ u64 wave_sum_u64(u64 v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

// LDS traffic between lanes of one wave needs no hardware barrier (a wave's LDS operations
// execute in order); this only stops the compiler from moving accesses across the point.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// Chunk states carry a 2-bit flag and a value in one 64-bit word (agent-scope relaxed
// atomics; no fences needed because the payload travels in the same word as the flag): first
// the chunk's hit total (flag AGG), later the inclusive prefix up to the chunk's end (flag
// INC).  A chunk's exclusive prefix is found by walking the states backwards, 64 chunks per
// step, summing totals until an inclusive prefix is met.  Waits are for chunks that are
// already being processed, and they are bounded by the spin limit.
__device__ __forceinline__ bool spin_once(u32& spins, u32 spin_limit, u32* d_status) {
  if (++spins > spin_limit) {  // give up, flag it, let everybody proceed
    if (lane_id() == 0) raise_status(d_status, FDY_ST_SPIN);
    return false;
  }
  __builtin_amdgcn_s_sleep(1);
  return true;
}

// Number of hits in all chunks before `chunk`.
__device__ __forceinline__ u64 chunk_exclusive_prefix(const u64* cstate, u32 chunk, u32 spin_limit,
                                                      u32* d_status) {
  const u32 l = lane_id();
  if (chunk == 0) return 0;
  u64 excl = 0;
  int pos = (int)chunk - 1;
  u32 spins = 0;
  for (;;) {
    const int idx = pos - (int)l;
    const u64 v = idx >= 0 ? ld_state(&cstate[idx]) : kFlagInc;  // before chunk 0: prefix 0
    const u32 flag = (u32)(v >> 62);
    const u64 inc_mask = ballot(flag == 2);
    const u64 empty_mask = ballot(flag == 0);
    const u32 first_inc = inc_mask ? (u32)__ffsll((long long)inc_mask) - 1 : 64;
    const u64 need = first_inc >= 63 ? ~0ull : ((2ull << first_inc) - 1);  // lanes 0..first_inc
    if (empty_mask & need) {
      if (!spin_once(spins, spin_limit, d_status)) break;
      continue;
    }
    excl += wave_sum_u64(((need >> l) & 1) ? (v & kValMask) : 0);
    if (first_inc < 64) break;
    pos -= 64;
  }
  return excl;
}

__device__ __forceinline__ u64 wave_incl_scan_u64(u64 v) {
  const u32 l = lane_id();
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const u64 o = __shfl_up(v, d);
    if (l >= (u32)d) v += o;
  }
  return v;
}

// A prepared table: magic and what it was made for (four 64-bit words), then the hierarchy,
// then the state.
struct PreparedHeader {
  u64 magic;
  u32 n_alloc, top_log2;
  u64 max_words;
  u64 table_ptr;
};
constexpr u64 kPreparedMagic = 0x3159445f4c424154ull;  // "TABL_DY1"
constexpr size_t kPreparedHeader = 256;

// Is the caller's prepared table one that was made for this table, this tuning and at least
// this many words?  (The host cannot look into device memory without a round trip.)
__device__ __forceinline__ bool prepared_ok(const ScanParams& p) {
  if (!p.prepared) return true;
  const u64 magic = p.prepared[0], sizes = p.prepared[1], max_words = p.prepared[2], table = p.prepared[3];
  return magic == kPreparedMagic && (u32)sizes == p.n_alloc && (u32)(sizes >> 32) == p.top_log2 &&
         p.n_words <= max_words && table == (u64)(uintptr_t)p.table;
}

// The scan's counters live in memory that outlasts the call when the caller prepared the table
// once (fdy_scan_table_prepare): then no launch zeroes them beforehand, and the last workgroup
// to finish leaves them as it found them, zero.  Called by one wave per workgroup, the one that
// wrote the workgroup's chunk states, after its last look-back: its state stores have been
// acknowledged (they are write-through, agent scope) before it counts itself done, so nothing
// of this launch can arrive after the reset.
__device__ __forceinline__ void finish_and_reset(const ScanParams& p) {
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  u32 n = 0;
  if (lane_id() == 0) n = __hip_atomic_fetch_add(p.done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  n = __shfl(n, 0);
  if (n + 1 != gridDim.x) return;
  for (u32 i = lane_id(); i < p.n_chunks; i += 64) st_state(&p.cstate[i], 0);
  if (lane_id() == 0) {
    __hip_atomic_store(p.ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p.done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// Level-0 keys are (base - span_lo) >> shift with the smallest shift that makes every key of
// the span fit key_bits bits (all-ones pads).  What the truncation leaves ambiguous is settled
// on the exact bases, so the shift affects speed only.  Keys are kept in 32 bits (key_bits =
// 31), or in 16 bits where LDS is needed for other things: then only a key's low half is
// stored, key_bits = 16 + bucket_log2 makes a bucket at most 2^16 key values wide, and the keys
// that a bucket's search compares all share their high half with the candidate.
__device__ __forceinline__ u32 key_shift_for(u64 span_len, u32 key_bits) {
  const u64 m = span_len - 1;
  const u32 bits = m ? 64u - (u32)__clzll((long long)m) : 0u;
  return bits > key_bits ? bits - key_bits : 0u;
}

// The level-0 key space is cut into 2^bucket_log2 equal buckets (key >> shift); the shift is the
// smallest that maps the span's largest key below the bucket count.
__device__ __forceinline__ u32 bucket_shift_for(u64 span_len, u32 key_shift, u32 bucket_log2) {
  const u64 max_key = (span_len - 1) >> key_shift;
  const u32 bits = max_key ? 64u - (u32)__clzll((long long)max_key) : 0u;
  return bits > bucket_log2 ? bits - bucket_log2 : 0u;
}

// Bytes that the level-0 keys take in LDS, in front of the bucket index (kept 16-byte aligned).
__device__ __host__ __forceinline__ size_t level0_key_bytes(u32 top_n, bool k16) {
  return k16 ? (((size_t)top_n * 2 + 15) & ~(size_t)15) : (size_t)top_n * 4;
}

struct Found {
  bool hit;
  u32 region;
  u64 offset;
  const u64* nb;  // where the region's new base is read from (launches with a base map)
};

// Level 1's choice (the last key of the node that is not above w: its place, and the key itself in gb)
// from the 32-byte form of a node: four 64-bit words {key 0; f1 f2 f3; f4 f5 f6;
// f7 s}, f_h = (key h - key 0) >> s in 21 bits each, s (6 bits, behind f7) the trailing zeros
// common to the seven distances.  False: the node is marked (last word ~0) because a distance
// does not fit or a key is padding; nothing is returned then.
constexpr u32 kCnodeField = (1u << 21) - 1;
__device__ __forceinline__ bool pick_cnode(const uint4 (&q)[2], u64 w, u32& at, u64& gb) {
  const u64 a0 = (u64)q[0].x | ((u64)q[0].y << 32), a1 = (u64)q[0].z | ((u64)q[0].w << 32);
  const u64 a2 = (u64)q[1].x | ((u64)q[1].y << 32), a3 = (u64)q[1].z | ((u64)q[1].w << 32);
  if (a3 == ~0ull) return false;
  const u32 s = (u32)(a3 >> 21) & 63u;
  const u64 x64 = (w - a0) >> s;  // floor: key h lies at or below w iff its distance <= x
  const u32 x = (x64 >> 32) ? 0xffffffffu : (u32)x64;
  const u32 f[8] = {0u,
                    (u32)a1 & kCnodeField,
                    (u32)(a1 >> 21) & kCnodeField,
                    (u32)(a1 >> 42) & kCnodeField,
                    (u32)a2 & kCnodeField,
                    (u32)(a2 >> 21) & kCnodeField,
                    (u32)(a2 >> 42) & kCnodeField,
                    (u32)a3 & kCnodeField};
  u32 d = 0;
  at = 0;
#pragma unroll
  for (int h = 1; h < 8; ++h)
    if (f[h] <= x) {
      at = h;
      d = f[h];
    }
  gb = a0 + ((u64)d << s);
  return true;
}

// The entry that w falls at or behind (entry index into n, exact base and size into e) from the
// 32-byte form of a table line: eight 32-bit words, distance >> sd in the high
// 12 bits and size >> ss in the low 20; the first entry's distance is 0 and its 12 bits hold
// sd (low six) and ss.  False: the line is marked (first word ~0).
__device__ __forceinline__ bool pick_cline(const uint4 (&q)[2], u64 w, u64 gb, u64& n, u64x2& e) {
  if (q[0].x == 0xffffffffu) return false;
  const u32 sd = (q[0].x >> 20) & 63u, ss = q[0].x >> 26;
  const u64 x = (w - gb) >> sd;
  // entry h lies at or below w iff its distance <= x, i.e. iff its whole word <= x's word with
  // all size bits set
  const u32 xt = x >= 4095u ? 0xffffffffu : (((u32)x << 20) | 0xfffffu);
  const u32 v[8] = {q[0].x & 0xfffffu, q[0].y, q[0].z, q[0].w, q[1].x, q[1].y, q[1].z, q[1].w};
  u32 pick = v[0], at = 0;
#pragma unroll
  for (int h = 1; h < 8; ++h)
    if (v[h] <= xt) {
      pick = v[h];
      at = h;
    }
  e.x = gb + ((u64)(pick >> 20) << sd);
  e.y = (u64)(pick & 0xfffffu) << ss;
  n = n * 8 + at;
  return true;
}

// Three dependent probes inside the table line itself: few registers, rarely taken.
__device__ __forceinline__ void probe_line(const ScanParams& p, u64 w, u64& n, u64x2& e) {
  n *= 8;
  e = *reinterpret_cast<const u64x2*>(&p.table[n]);
#pragma unroll 1
  for (u32 step = 4; step; step >>= 1) {
    if (n + step < p.n_alloc) {
      const u64x2 q = *reinterpret_cast<const u64x2*>(&p.table[n + step]);
      if (q.x <= w) {
        n += step;
        e = q;
      }
    }
  }
}

// The 64-byte node or line for the rare candidate whose compact node or line is marked: the
// place is counted (keys and distances ascend) and the chosen value read again, which needs
// no node held in registers beside the interleaved chains.
__device__ __forceinline__ u32 probe_node(const u64* m, u64 first_key, u64 w, u64& gb) {
  u32 at = 0;
#pragma unroll
  for (int h = 1; h < 8; ++h) at += m[first_key + h] <= w ? 1u : 0u;
  gb = m[first_key + at];
  return at;
}

__device__ __forceinline__ bool probe_wide_line(const uint4* leaf, u64 w, u64 gb, u64& n, u64x2& e) {
  const uint4* line = leaf + n * 4;
  const uint4 q0 = line[0];
  if (q0.x == 0xffffffffu) return false;
  const uint4 q1 = line[1], q2 = line[2], q3 = line[3];
  const u32 sh = q0.x;
  const u64 x = (w - gb) >> sh;
  const u32 at = ((u64)q0.z <= x ? 1u : 0u) + ((u64)q1.x <= x ? 1u : 0u) + ((u64)q1.z <= x ? 1u : 0u) +
                 ((u64)q2.x <= x ? 1u : 0u) + ((u64)q2.z <= x ? 1u : 0u) + ((u64)q3.x <= x ? 1u : 0u) +
                 ((u64)q3.z <= x ? 1u : 0u);
  const uint2 dz = reinterpret_cast<const uint2*>(line)[at];
  e.x = gb + ((u64)(at ? dz.x : 0u) << sh);
  e.y = (u64)dz.y << sh;
  n = n * 8 + at;
  return true;
}

// Whether a compact array is worth reading for this table: where most nodes are marked a
// candidate would pay the compact fetch and then the wide one, so the choice is made per
// table, from 64 evenly spaced nodes (all lanes of the wave take part).
__device__ __forceinline__ bool mostly_packed(const uint4* arr, u32 n_nodes, bool node_form) {
  if (!arr || !n_nodes) return false;
  const u64 i = ((u64)lane_id() * n_nodes) >> 6;
  const uint4 q = arr[i * 2 + (node_form ? 1 : 0)];
  const bool marked = node_form ? (q.z & q.w) == 0xffffffffu : q.x == 0xffffffffu;
  return __popcll(ballot(marked)) <= 16;
}

constexpr u32 kUseCmid = 1u << 16, kUseCleaf = 1u << 17;  // flags that travel with the shifts

// Interval search for N candidates per lane at once (each w lies inside the table's span).
// The N chains are independent; writing every step for all of them lets their LDS and
// global round trips overlap, which is what the dependent steps of one chain cannot do.
template <int N, bool kK16 = false, bool kRecords = kK16>
__device__ __forceinline__ void search(const ScanParams& p, const void* top_v, u64 span_lo, u32 shifts,
                                       const u64 (&w)[N], Found (&f)[N], u32& marked) {
  typedef typename std::conditional<kK16, unsigned short, u32>::type key_t;
  const key_t* top = reinterpret_cast<const key_t*>(top_v);
  const u32 key_shift = shifts & 0xffu, bucket_shift = (shifts >> 8) & 0xffu;
  const uint4* cmid = (shifts & kUseCmid) ? p.cmid : nullptr;
  const uint4* cleaf = (shifts & kUseCleaf) ? p.cleaf : nullptr;
  u32 kw[N], i[N];
  u64 n[N];
#pragma unroll
  for (int c = 0; c < N; ++c) {
    kw[c] = (u32)((w[c] - span_lo) >> key_shift);
    i[c] = 0;
  }
  // level 0: a bucket index first (which keys can the answer be among: two adjacent 16-bit
  // reads), then a binary search among just those.  With about one key per bucket that is 3-5
  // LDS reads in 2-4 dependent steps, where a search over all 16,384 keys takes 14 (or 21 in
  // 7 steps, 4-ary): level 0 was 27 % of the kernel's time, most of it LDS bank conflicts of
  // 64 lanes reading random keys.  Clustered tables degrade towards the plain binary search.
  {
    const unsigned short* bst = reinterpret_cast<const unsigned short*>(
        reinterpret_cast<const unsigned char*>(top_v) + level0_key_bytes(p.top_n, kK16));
    u32 lo[N], hi[N], kc[N];  // kc: the candidate's key as the stored keys compare with it
#pragma unroll
    for (int c = 0; c < N; ++c) {
      const u32 bk = kw[c] >> bucket_shift;
      lo[c] = bst[bk];
      hi[c] = bst[bk + 1];
      kc[c] = kK16 ? (kw[c] & 0xffffu) : kw[c];
    }
    for (;;) {
      bool open = false;
#pragma unroll
      for (int c = 0; c < N; ++c) open = open || lo[c] < hi[c];
      if (!ballot(open)) break;
      u32 k[N];
#pragma unroll
      for (int c = 0; c < N; ++c) k[c] = lo[c] < hi[c] ? (u32)top[(lo[c] + hi[c]) >> 1] : 0u;
#pragma unroll
      for (int c = 0; c < N; ++c)
        if (lo[c] < hi[c]) {
          const u32 mid = (lo[c] + hi[c]) >> 1;
          if (k[c] <= kc[c]) lo[c] = mid + 1;
          else hi[c] = mid;
        }
    }
#pragma unroll
    for (int c = 0; c < N; ++c) i[c] = lo[c] - 1;  // keys not above kw, minus one; key 0 is 0
#pragma unroll
    for (int c = 0; c < N; ++c) kw[c] = kc[c];
  }
#pragma unroll
  for (int c = 0; c < N; ++c) {
    n[c] = i[c];  // node index at level `levels`: covers table entries [n * 8^levels, ...)
    if ((u32)top[i[c]] == kw[c]) {
      // equal keys: the sampled base may still lie above w; settle it on exact bases (16-bit
      // keys of another bucket may look equal too: the settling then changes nothing)
      const u32 sh = 3 * p.levels + p.f0_log2;
      while (n[c] > 0 && p.table[n[c] << sh].base > w[c]) --n[c];
    }
  }
  if (p.f0_log2) {
    // a level-0 key spans 2^f0_log2 nodes of the first packed level: 1-2 binary steps there
    const u64* m = p.mid[p.levels - 1];
#pragma unroll
    for (int c = 0; c < N; ++c) n[c] <<= p.f0_log2;
    for (u32 step = 1u << (p.f0_log2 - 1); step; step >>= 1) {
#pragma unroll
      for (int c = 0; c < N; ++c)
        if (m[n[c] + step] <= w[c]) n[c] += step;
    }
  }
  // Packed levels: the whole 64-byte node of 8 keys per candidate, fetched with four
  // independent 16-byte loads (requests to one line merge, so this costs the memory system
  // about what a single probe does, where three dependent probes cost three round trips and
  // three requests: the vector L1 is far too small to keep a node between two probes of the
  // same lane).  The child is the last key not above w: keys are ascending, padded with ~0,
  // and the first key of the node is known not to exceed w.  Level 1 is read through its
  // 32-byte copy when the table has one that mostly packs: two loads per candidate instead of
  // four (a lane's load costs the vector memory unit its turn whether or not the line merges).
  u64 gb[N];  // exact base of the first entry of the candidate's table line (level 1's key)
#pragma unroll
  for (int c = 0; c < N; ++c) gb[c] = 0;
  for (int j = (int)p.levels - 1; j >= 1; --j) {
    const u64* m = p.mid[j - 1];
    if (j == 1 && cmid) {
      uint4 cq[N][2];
#pragma unroll
      for (int c = 0; c < N; ++c) {
        cq[c][0] = cmid[n[c] * 2];
        cq[c][1] = cmid[n[c] * 2 + 1];
      }
      __builtin_amdgcn_sched_barrier(0);  // every chain's node is requested before the first is used
#pragma unroll
      for (int c = 0; c < N; ++c) {
        n[c] *= 8;
        u32 at;
        const bool packed = pick_cnode(cq[c], w[c], at, gb[c]);
        if (!packed) at = probe_node(m, n[c], w[c], gb[c]);  // a marked node
        marked += (u32)__popcll(ballot(!packed));
        n[c] += at;
      }
      continue;
    }
    u64x2 k[N][4];
#pragma unroll
    for (int c = 0; c < N; ++c) {
      n[c] *= 8;
#pragma unroll
      for (int h = 0; h < 4; ++h) k[c][h] = *reinterpret_cast<const u64x2*>(&m[n[c] + 2 * h]);
    }
    // every chain's node is requested before the first one is looked at (left to itself the
    // scheduler sinks each chain's loads next to their use and the round trips line up)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < N; ++c) {
      u32 at = 0;
      gb[c] = k[c][0].x;
#pragma unroll
      for (int h = 1; h < 8; ++h) {
        const u64 key = (h & 1) ? k[c][h >> 1].y : k[c][h >> 1].x;
        if (key <= w[c]) {
          at = h;
          gb[c] = key;
        }
      }
      n[c] += at;
    }
  }
  // Leaf: 8 consecutive entries of the table.  Large tables are not read directly: a packed
  // copy holds each line in 64 bytes, {base - first base of the line, size} in 32 bits each
  // after a shift by the line's common trailing zeros,
  // which halves what the candidate has to pull through the memory fabric (this fetch is what
  // bounds the scan when the table outgrows L2), and where the lines mostly allow it a
  // compact copy holds them in 32 bytes (12-bit distances, 20-bit sizes, a shift for each),
  // which halves it again and lets most of the copy stay in an XCD's L2.  A line whose values
  // do not fit the compact form is marked there and read from the 64-byte copy; one that does
  // not fit that either, and the last, partial line, are marked and read from the table
  // itself; so are all lines of small tables, which stay in L2 anyway.  Either way the whole
  // line is fetched at once.
  u64x2 e[N];
  const u64* nbl[N];  // base of the new-base array to index with the region: the line's own copy, if any
#pragma unroll
  for (int c = 0; c < N; ++c) nbl[c] = nullptr;
  if (p.levels == 0) {
#pragma unroll
    for (int c = 0; c < N; ++c) e[c] = *reinterpret_cast<const u64x2*>(&p.table[n[c]]);
  } else if (cleaf) {
    // With a base map the compact line comes from a copy that keeps the eight regions' new
    // bases in the same 128-byte memory line: the hit's new base, asked for a round trip later,
    // is then found in the L2 that has just fetched the line (from the base map itself, 8 bytes
    // at a random place of 8 MiB, three out of four such requests went on to the memory side).
    const uint4* lm = kRecords ? p.leafmap : nullptr;
    uint4 cq[N][2];
#pragma unroll
    for (int c = 0; c < N; ++c) {
      cq[c][0] = lm ? lm[n[c] * 8] : cleaf[n[c] * 2];
      cq[c][1] = lm ? lm[n[c] * 8 + 1] : cleaf[n[c] * 2 + 1];
      nbl[c] = lm ? reinterpret_cast<const u64*>(lm + n[c] * 8 + 2) - n[c] * 8 : nullptr;
    }
    __builtin_amdgcn_sched_barrier(0);  // every chain's line is requested before the first is used
#pragma unroll
    for (int c = 0; c < N; ++c) {
      const bool packed = pick_cline(cq[c], w[c], gb[c], n[c], e[c]);
      if (!packed) nbl[c] = nullptr;
      // a marked line: the 64-byte copy, then the table
      if (!packed && !probe_wide_line(p.leaf, w[c], gb[c], n[c], e[c])) probe_line(p, w[c], n[c], e[c]);
      marked += (u32)__popcll(ballot(!packed));
    }
  } else {
    uint4 ql[N][4];
    if (p.leaf) {
#pragma unroll
      for (int c = 0; c < N; ++c) {
#pragma unroll
        for (int h = 0; h < 4; ++h) ql[c][h] = p.leaf[n[c] * 4 + h];
      }
      __builtin_amdgcn_sched_barrier(0);  // every chain's line is requested before the first is used
    }
#pragma unroll
    for (int c = 0; c < N; ++c) {
      bool exact = true;
      if (p.leaf) {
        const uint4 (&q)[4] = ql[c];
        if (q[0].x != 0xffffffffu) {
          exact = false;
          const u32 sh = q[0].x;  // the line's shift (at most 31); the first entry's distance is 0
          const u64 x = (w[c] - gb[c]) >> sh;  // floor: entry h lies at or below w iff its distance <= x
          u32 d = 0, z = q[0].y, at = 0;
#pragma unroll
          for (int h = 1; h < 8; ++h) {
            const u32 dh = (h & 1) ? q[h >> 1].z : q[h >> 1].x;
            const u32 zh = (h & 1) ? q[h >> 1].w : q[h >> 1].y;
            if ((u64)dh <= x) {
              d = dh;
              z = zh;
              at = h;
            }
          }
          e[c].x = gb[c] + ((u64)d << sh);
          e[c].y = (u64)z << sh;
          n[c] = n[c] * 8 + at;
        }
      }
      // one candidate after the other (the loads in flight per lane already cover the
      // latency; more would only cost registers)
      if (exact) probe_line(p, w[c], n[c], e[c]);
      __builtin_amdgcn_sched_barrier(0);  // keep the next candidate's loads behind this one's
    }
  }
#pragma unroll
  for (int c = 0; c < N; ++c) {
    f[c].offset = w[c] - e[c].x;
    f[c].region = (u32)n[c];
    f[c].hit = f[c].offset < e[c].y;
    f[c].nb = (nbl[c] ? nbl[c] : p.new_base) + n[c];
  }
}

// Outcome of the span pre-filter for one sub-tile as a wave holds it (8 words per lane): which
// words are candidates, and each candidate's rank in word order (load k, lane, half).
// Stages the level-0 keys and the bucket index in LDS with 16-byte copies.  Both arrays are
// padded to 256 bytes in the workspace and to 16 bytes in LDS, so whole 16-byte pieces can be
// copied past their last entry; a top level of two keys (8 bytes) is copied key by key.
__device__ __forceinline__ void stage_level0(const ScanParams& p, void* top_v, unsigned short* bst, u32 n_bst,
                                             bool k16 = false) {
  const u32 tid = threadIdx.x;
  u32* top = reinterpret_cast<u32*>(top_v);
  if (k16) {  // 16-bit keys: top_n >= 2 of them, padded to 16 bytes in both places
    const uint4* src = reinterpret_cast<const uint4*>(p.top);
    uint4* dst = reinterpret_cast<uint4*>(top);
    for (u32 i = tid; i < (p.top_n * 2 + 15) / 16; i += kBlock) dst[i] = src[i];
    const uint4* bsrc = reinterpret_cast<const uint4*>(p.bstart);
    uint4* bdst = reinterpret_cast<uint4*>(bst);
    for (u32 i = tid; i < (n_bst * 2 + 15) / 16; i += kBlock) bdst[i] = bsrc[i];
  } else if (p.top_n >= 4) {
    const uint4* src = reinterpret_cast<const uint4*>(p.top);
    uint4* dst = reinterpret_cast<uint4*>(top);
    for (u32 i = tid; i < p.top_n / 4; i += kBlock) dst[i] = src[i];
    const uint4* bsrc = reinterpret_cast<const uint4*>(p.bstart);
    uint4* bdst = reinterpret_cast<uint4*>(bst);
    for (u32 i = tid; i < (n_bst * 2 + 15) / 16; i += kBlock) bdst[i] = bsrc[i];
  } else {
    for (u32 i = tid; i < p.top_n; i += kBlock) top[i] = p.top[i];
    for (u32 i = tid; i < n_bst; i += kBlock) bst[i] = p.bstart[i];
  }
}

struct Filt {
  bool c[kWpl];
  u32 crank[kWpl];
  u32 Q;
};

// kHalf: the array is read as 32-bit units and position q stands for the 64-bit value whose low
// half is unit q and whose high half is unit q + 1 (pointers at 4-byte alignment inside packed
// structures); p.n_words is then the number of positions, one less than the number of units.
// A lane still takes 16-byte pieces, four positions each, and gets the unit that follows its
// piece from the next lane (the last lane from the next piece, or from behind the sub-tile).
template <bool kHalf>
__device__ __forceinline__ void load_words(const ScanParams& p, u32 sub, u64 span_lo, u64 (&w)[kWpl]) {
  const u32 lane = lane_id();
  const u64 wbase = (u64)sub * kSub;
  if constexpr (kHalf) {
    static_assert(kWpl == 8, "two 16-byte pieces of four positions per lane");
    const u32* h = reinterpret_cast<const u32*>(p.words);
    if (wbase + kSub <= p.n_words) {  // all 512 positions exist, hence units wbase .. wbase + 512
      typedef u32 v4u32 __attribute__((ext_vector_type(4)));
      v4u32 v[2];
#pragma unroll
      for (int k = 0; k < 2; ++k)
        v[k] = __builtin_nontemporal_load(reinterpret_cast<const v4u32*>(h + wbase + (k * 64 + lane) * 4));
      const u32 behind = h[wbase + kSub];
      u32 nx[2];
      nx[0] = __shfl_down(v[0].x, 1);
      nx[1] = __shfl_down(v[1].x, 1);
      const u32 first1 = __shfl(v[1].x, 0);
      if (lane == 63) {
        nx[0] = first1;
        nx[1] = behind;
      }
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        w[4 * k + 0] = (u64)v[k].x | ((u64)v[k].y << 32);
        w[4 * k + 1] = (u64)v[k].y | ((u64)v[k].z << 32);
        w[4 * k + 2] = (u64)v[k].z | ((u64)v[k].w << 32);
        w[4 * k + 3] = (u64)v[k].w | ((u64)nx[k] << 32);
      }
    } else {  // the ragged tail, and sub-tiles past the end
#pragma unroll
      for (int r = 0; r < kWpl; ++r) {
        const u64 q = wbase + ((r >> 2) * 64 + lane) * 4 + (r & 3);
        w[r] = q < p.n_words ? ((u64)h[q] | ((u64)h[q + 1] << 32)) : span_lo - 1;  // outside the span
      }
    }
  } else if (wbase + kSub <= p.n_words) {
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      // streamed once: non-temporal, so that the table levels keep their place in L2
      typedef u64 v2u64 __attribute__((ext_vector_type(2)));
      const v2u64 v =
          __builtin_nontemporal_load(reinterpret_cast<const v2u64*>(p.words + wbase + (k * 64 + lane) * 2));
      w[2 * k] = v.x;
      w[2 * k + 1] = v.y;
    }
  } else {  // the ragged tail, and sub-tiles past the end (no word is read, none is a candidate)
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const u64 idx = wbase + (k * 64 + lane) * 2;
      w[2 * k] = idx < p.n_words ? p.words[idx] : span_lo - 1;  // outside the span
      w[2 * k + 1] = idx + 1 < p.n_words ? p.words[idx + 1] : span_lo - 1;
    }
  }
}

// Register r of a lane holds position (r / kPer * 64 + lane) * kPer + r % kPer of the sub-tile,
// kPer = 2 words per 16-byte piece, or 4 positions per piece when reading 32-bit units.
template <bool kHalf>
__device__ __forceinline__ u32 pos_in_sub(int r, u32 lane) {
  constexpr int kPer = kHalf ? 4 : 2;
  return ((u32)(r / kPer) * 64 + lane) * kPer + (u32)(r % kPer);
}

template <bool kHalf>
__device__ __forceinline__ void filter_words(const u64 (&w)[kWpl], Filt& t, u64 span_lo, u64 span_len) {
  constexpr int kPer = kHalf ? 4 : 2;
  const u64 lt = lanemask_lt();
  t.Q = 0;
#pragma unroll
  for (int k = 0; k < kWpl / kPer; ++k) {
    u32 below = t.Q, all = 0;  // candidates of lower lanes in this piece row; of all lanes
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      t.c[kPer * k + j] = (w[kPer * k + j] - span_lo) < span_len;
      const u64 b = ballot(t.c[kPer * k + j]);
      below += __popcll(b & lt);
      all += __popcll(b);
    }
    u32 own = 0;  // this lane's earlier candidates of the piece
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      t.crank[kPer * k + j] = below + own;
      own += t.c[kPer * k + j] ? 1u : 0u;
    }
    t.Q += all;
  }
}

// Candidates with rank in [win, win + wn) go to queue slots qoff + [0, wn); the index stored
// with each is its word's distance from word 0 of the sub-tile `row` places before this one.
// kValues false: only the indices are queued (the values are found through them, in the
// wave's copy of its words in LDS).
template <bool kHalf, bool kValues = true>
__device__ __forceinline__ void enqueue(const u64 (&w)[kWpl], const Filt& t, u32 row, u32 win, u32 wn,
                                        u32 qoff, u64* qw, unsigned short* qi) {
  const u32 lane = lane_id();
  wave_lds_fence();
#pragma unroll
  for (int r = 0; r < kWpl; ++r)
    if (t.c[r] && t.crank[r] - win < wn) {  // unsigned: also false below the window
      if constexpr (kValues) qw[qoff + t.crank[r] - win] = w[r];
      qi[qoff + t.crank[r] - win] = (unsigned short)(row * kSub + pos_in_sub<kHalf>(r, lane));
    }
  wave_lds_fence();
}

// The wave's copy of a sub-tile in LDS (ordered scan with rebased output): written as loaded,
// 16 bytes per lane and load, so that word i of the sub-tile lies at index i.
__device__ __forceinline__ void stash_words(u64* stash, const u64 (&w)[kWpl]) {
  const u32 lane = lane_id();
#pragma unroll
  for (int k = 0; k < kLoads; ++k) {
    u64x2 v;
    v.x = w[2 * k];
    v.y = w[2 * k + 1];
    *reinterpret_cast<u64x2*>(stash + (k * 64 + lane) * 2) = v;
  }
}

// ... and back from LDS to the output array, whole 16-byte pieces, non-temporally (written once).
__device__ __forceinline__ void unstash_words(const ScanParams& p, u32 sub, const u64* stash) {
  typedef u64 v2u64 __attribute__((ext_vector_type(2)));
  const u32 lane = lane_id();
  const u64 wbase = (u64)sub * kSub;
  if (wbase + kSub <= p.n_words) {
    u64x2 v[kLoads];
#pragma unroll
    for (int k = 0; k < kLoads; ++k) v[k] = *reinterpret_cast<const u64x2*>(stash + (k * 64 + lane) * 2);
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      v2u64 o;
      o.x = v[k].x;
      o.y = v[k].y;
      __builtin_nontemporal_store(o, reinterpret_cast<v2u64*>(p.out + wbase + (k * 64 + lane) * 2));
    }
  } else {
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const u32 i = (k * 64 + lane) * 2;
      if (wbase + i < p.n_words) p.out[wbase + i] = stash[i];
      if (wbase + i + 1 < p.n_words) p.out[wbase + i + 1] = stash[i + 1];
    }
  }
}

// A sub-tile's words as the lanes hold them, to the output: the 16-byte stores a copy would use.
// kNt: non-temporal (written once, not touched again by this kernel).
template <bool kNt>
__device__ __forceinline__ void store_words(const ScanParams& p, u32 sub, const u64 (&w)[kWpl]) {
  typedef u64 v2u64 __attribute__((ext_vector_type(2)));
  const u32 lane = lane_id();
  const u64 wbase = (u64)sub * kSub;
  if (wbase + kSub <= p.n_words) {
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      v2u64 v;
      v.x = w[2 * k];
      v.y = w[2 * k + 1];
      v2u64* dst = reinterpret_cast<v2u64*>(p.out + wbase + (k * 64 + lane) * 2);
      if constexpr (kNt) __builtin_nontemporal_store(v, dst);
      else *dst = v;
    }
  } else {
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const u64 idx = wbase + (k * 64 + lane) * 2;
      if (idx < p.n_words) p.out[idx] = w[2 * k];
      if (idx + 1 < p.n_words) p.out[idx + 1] = w[2 * k + 1];
    }
  }
}

__device__ __forceinline__ void store_reloc(const ScanParams& p, u64 at, u32 word, u32 region, u64 offset) {
  if (at < p.capacity) {
    fdy_reloc o;
    o.word = word;
    o.region = region;
    o.offset = offset;
    *reinterpret_cast<uint4*>(&p.relocs[at]) = *reinterpret_cast<const uint4*>(&o);
  }
}

// Dense sub-tile (its wave's group holds more candidates than the register-resident path
// keeps): windows of queue size, searched one round at a time; the hits go to dst[0 ...) as
// complete entries in word order (the wave's staging area: the output position is not known
// yet).  Returns hits.
// kStash: qw is the wave's LDS copy of this sub-tile; candidates are read from it through their
// indices and a hit's word is replaced by its rebased value there.
// What becomes of the hits: kDenseStage - complete entries to dst[0 ...) (staging);
// kDenseCount - nothing, they are only counted (no staging area: the group is searched again
// when its position is known); kDenseWrite - that second search: entries to the relocation
// table from position dst_pos on, within its capacity.
enum { kDenseStage = 0, kDenseCount = 1, kDenseWrite = 2 };
template <bool kHalf, bool kK16, bool kStash, int kMode>
__device__ u64 dense_pass(const ScanParams& p, const u64 (&w)[kWpl], const Filt& t, const void* top,
                          u64 span_lo, u32 shifts, u64* qw, unsigned short* qi, u64 wbase, fdy_reloc* dst,
                          u64 dst_pos, u32& marked) {
  const u32 lane = lane_id();
  const u64 lt = lanemask_lt();
  u64 H = 0;
  for (u32 win = 0; win < t.Q; win += kQcap) {
    const u32 wn = t.Q - win < (u32)kQcap ? t.Q - win : (u32)kQcap;
    enqueue<kHalf, !kStash>(w, t, 0, win, wn, 0, qw, qi);
    for (u32 q0 = 0; q0 < wn; q0 += 64) {
      const u32 q = q0 + lane;
      const bool valid = q < wn;
      const u64 wv[1] = {valid ? qw[kStash ? (u32)qi[q] : q] : span_lo};
      Found f[1];
      search<1, kK16>(p, top, span_lo, shifts, wv, f, marked);
      const bool hit = valid && f[0].hit;
      const u64 b = ballot(hit);
      if (hit) {
        fdy_reloc o;
        o.word = (u32)(wbase + qi[q]);
        o.region = f[0].region;
        o.offset = f[0].offset;
        if constexpr (kMode == kDenseStage)
          *reinterpret_cast<uint4*>(&dst[H + __popcll(b & lt)]) = *reinterpret_cast<const uint4*>(&o);
        if constexpr (kMode == kDenseWrite) store_reloc(p, dst_pos + H + __popcll(b & lt), o.word, o.region, o.offset);
        if constexpr (kStash) qw[qi[q]] = *f[0].nb + o.offset;
      }
      H += __popcll(b);
    }
  }
  return H;
}

// Searches queue rounds [R0, R0 + N) (64 entries each), N per lane in flight at once; region
// (kMiss for "no hit") and offset stay in the caller's registers, round k's lane l holding the
// result of queue slot 64 k + l.
template <int N, int R0, int kGR, bool kOut>
__device__ __forceinline__ void run_rounds(const ScanParams& p, const void* top, u64 span_lo, u32 shifts,
                                           u64* qw, u32 Q, u32 (&reg)[kGR], u64 (&off)[kGR], u64& H, u32& marked,
                                           const unsigned short* qi) {
  static_assert(R0 + N <= kGR, "rounds");
  const u32 lane = lane_id();
  u64 wv[N];
  Found f[N];
  bool valid[N];
  u32 at[N];  // kOut: where the candidate lies in the wave's LDS copy of the group's words
#pragma unroll
  for (int r = 0; r < N; ++r) {
    valid[r] = (R0 + r) * 64 + lane < Q;
    at[r] = kOut && valid[r] ? (u32)qi[(R0 + r) * 64 + lane] : (u32)((R0 + r) * 64 + lane);
    wv[r] = valid[r] ? qw[at[r]] : span_lo;
  }
  search<N, kOut>(p, top, span_lo, shifts, wv, f, marked);
#pragma unroll
  for (int r = 0; r < N; ++r) {
    const bool hit = valid[r] && f[r].hit;
    reg[R0 + r] = hit ? f[r].region : kMiss;
    off[R0 + r] = f[r].offset;
    H += __popcll(ballot(hit));
  }
  if constexpr (kOut) {
    // a hit's word in the LDS copy becomes its rebased value; the copy goes out as a whole later
    u64 nb[N];
#pragma unroll
    for (int r = 0; r < N; ++r) nb[r] = reg[R0 + r] != kMiss ? *f[r].nb : 0;
#pragma unroll
    for (int r = 0; r < N; ++r)
      if (reg[R0 + r] != kMiss) qw[at[r]] = nb[r] + off[R0 + r];
  }
}

// Rounds [R0, R0 + 3) as far as there are candidates, with as many chains per lane as rounds.
template <int R0, int kGR, bool kOut>
__device__ __forceinline__ void run_group(const ScanParams& p, const void* top, u64 span_lo, u32 shifts,
                                          u64* qw, u32 Q, u32 (&reg)[kGR], u64 (&off)[kGR], u64& H, u32& marked,
                                          const unsigned short* qi) {
  if constexpr (R0 + 3 <= kGR) {
    const u32 nr = (Q + 63) >> 6;
    if (nr >= (u32)R0 + 3) run_rounds<3, R0, kGR, kOut>(p, top, span_lo, shifts, qw, Q, reg, off, H, marked, qi);
    else if (nr == (u32)R0 + 2) run_rounds<2, R0, kGR, kOut>(p, top, span_lo, shifts, qw, Q, reg, off, H, marked, qi);
    else if (nr == (u32)R0 + 1) run_rounds<1, R0, kGR, kOut>(p, top, span_lo, shifts, qw, Q, reg, off, H, marked, qi);
  }
}

// Results of one wave for one chunk, register-resident but for the candidates' word indices,
// which stay where the queue put them in LDS (two halves, used by alternate rounds).  The wave's sub-tiles come in kGroups
// groups of kG consecutive ones; the candidates of a group share one queue and are searched
// in dense rounds of 64, up to kG * kRegRounds rounds per group.
template <int kGroups, int kG>
struct RoundResults {
  static constexpr int kGR = kG * kRegRounds;
  u32 reg[kGroups][kGR];  // region, kMiss for "no hit"
  u64 off[kGroups][kGR];  // offset inside the region
  u32 b;                  // which half of the wave's index queues belongs to this chunk
  u32 Q[kGroups];         // candidates of the group (dense path if above the register limit)
  u32 H[kGroups];         // hits of the group
  u64 cnt_incl;           // lane l: hits of the chunk's (group, wave) units 0..l
  u32 base;               // first sub-tile of the chunk
};

// Ordered write of one chunk's hits of this wave, given the chunk's exclusive prefix.
// The staging area of a wave's group: entries of the dense groups of chunk parity b.  A unit
// (group, wave) has room for one entry per word it covers.
template <int kGroups, int kG>
__device__ __forceinline__ fdy_reloc* stage_of(const ScanParams& p, u32 b, int g) {
  constexpr u32 kUnitWords = kG * kSub, kUnits = kGroups * kWaves;
  const u32 wave = threadIdx.x >> 6;
  return p.stage + ((u64)blockIdx.x * 2 + b) * (kUnits * kUnitWords) + (u64)(g * kWaves + wave) * kUnitWords;
}

// A dense group without a staging area is searched a second time here, from the words in
// memory (scratch: the wave's value queue qw, idle between rounds, and the group's own index
// queue, which a dense group does not use).
template <int kGroups, int kG, bool kHalf, bool kK16, bool kStaged>
__device__ __forceinline__ void write_round(const ScanParams& p, const RoundResults<kGroups, kG>& r,
                                            u64 chunk_excl, unsigned short* qi_all, const void* top, u64 span_lo,
                                            u64 span_len, u32 shifts, u64* qw, u32& marked) {
  constexpr int kGR = kG * kRegRounds;
  const u32 wave = threadIdx.x >> 6;
  const u64 lt = lanemask_lt();
#pragma unroll
  for (int g = 0; g < kGroups; ++g) {
    const u32 first_sub = r.base + (g * kWaves + wave) * kG;
    u64 pos = chunk_excl + __shfl(r.cnt_incl, g * kWaves + wave) - r.H[g];
    unsigned short* qi = qi_all + (r.b * kGroups + g) * (kG * kQcap);
    if (r.Q[g] <= (u32)(kGR * 64)) {
      const u64 wbase = (u64)first_sub * kSub;
#pragma unroll
      for (int k = 0; k < kGR; ++k) {
        const bool hit = r.reg[g][k] != kMiss;
        const u64 bl = ballot(hit);
        if (hit)
          store_reloc(p, pos + __popcll(bl & lt), (u32)(wbase + qi[k * 64 + lane_id()]), r.reg[g][k], r.off[g][k]);
        pos += __popcll(bl);
      }
    } else if constexpr (!kStaged) {
      u64 H = 0;
      for (int row = 0; row < kG; ++row) {
        u64 dw[kWpl];
        Filt t;
        load_words<kHalf>(p, first_sub + row, span_lo, dw);
        filter_words<kHalf>(dw, t, span_lo, span_len);
        H += dense_pass<kHalf, kK16, false, kDenseWrite>(p, dw, t, top, span_lo, shifts, qw, qi,
                                                         (u64)(first_sub + row) * kSub, nullptr, pos + H, marked);
      }
    } else {
      // a dense group: its entries wait in the wave's staging area, complete and in word
      // order, written a round ago by other lanes of this wave, through the same vector L1
      // (workgroup scope: a wider fence would write back and invalidate the whole L2)
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      const fdy_reloc* src = stage_of<kGroups, kG>(p, r.b, g);
      for (u32 i = lane_id(); i < r.H[g]; i += 64) {
        const uint4 v = *reinterpret_cast<const uint4*>(&src[i]);
        if (pos + i < p.capacity) *reinterpret_cast<uint4*>(&p.relocs[pos + i]) = v;
      }
    }
  }
}

// kOut: the scan also writes the rebased copy of the words (p.out, p.new_base).  A wave then
// keeps the words of its group in LDS instead of queueing the candidates' values (the queue
// holds their indices only and the search reads them through those); a hit's word is
// replaced there by new_base[region] + offset right after the search, and the group goes out
// as whole sub-tiles with the stores a copy would use.  (Copying the words to the output when
// they are loaded and storing the hits' values over them afterwards was measured at twice the
// time: by then the lines have left the L2, and 13 M scattered 8-byte stores into memory cost
// more than the whole scan.)  The 64 KiB this takes come from the level-0 keys, which such a
// launch keeps in 16 bits each, and from half of the bucket index.
// kStaged: the workspace holds a staging area for dense groups.  The other variant searches
// them twice and carries that second search's code.  (One kernel that chose between the two
// at run time was measured 3 to 5 % slower than either, on inputs without a single dense
// group: this kernel's time moves by that much with the size and layout of its code.)
template <int kGroups, int kG, bool kHalf, bool kOut, bool kStaged>
__global__ __launch_bounds__(kBlock) void scan_kernel(ScanParams p) {
  constexpr int kUnits = kGroups * kWaves;  // (group, wave) units of a chunk, in word order
  constexpr int kChunk = kUnits * kG;       // sub-tiles a workgroup draws per ticket
  constexpr int kGR = kG * kRegRounds;
  constexpr u32 kQwave = kG * kQcap;        // queue entries per wave
  static_assert(kUnits <= 64 && kG * kSub <= 65536, "a chunk's counts fit one wave; 16-bit queue indices");
  static_assert(!(kOut && kHalf), "the rebased output exists for aligned words only");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  __shared__ u32 s_next[2];         // first sub-tile of the chunk two rounds ahead, per round parity
  __shared__ u32 s_cnt[2][kUnits];  // hit counts of the chunk's units
  __shared__ u64 s_excl[2];         // previous chunk's exclusive prefix, from the closer wave
  void* top = smem_raw;  // [top_n] keys of 32 (kOut: 16) bits, then the bucket index behind them
  unsigned short* bst = reinterpret_cast<unsigned short*>(smem_raw + level0_key_bytes(p.top_n, kOut));  // [n_buckets + 1]
  const u32 n_bst = (1u << p.bucket_log2) + 1;
  unsigned char* qbase = smem_raw + level0_key_bytes(p.top_n, kOut) + (((size_t)n_bst * 2 + 15) & ~(size_t)15);
  const u32 tid = threadIdx.x;
  const u32 lane = tid & 63;
  const u32 wave = tid >> 6;
  // candidate values (kOut: the words of the wave's group, kG sub-tiles)
  constexpr u32 kVwave = kOut ? (u32)(kG * kSub) : kQwave;
  u64* qw = reinterpret_cast<u64*>(qbase) + wave * kVwave;
  unsigned short* qi_all = reinterpret_cast<unsigned short*>(qbase + (size_t)kWaves * kVwave * 8) +
                           wave * (2 * kGroups * kQwave);  // word indices: [round parity][group][slot]
  const bool closer = wave == kWaves - 1;  // one wave per workgroup speaks for the chunk
  if (!prepared_ok(p)) {  // every workgroup sees the same: nothing is read or written
    if (blockIdx.x == 0 && tid == 0) raise_status(p.d_status, FDY_ST_BAD_PREPARED);
    return;
  }

  // Chunks are drawn two rounds ahead, so that a round knows where the next one reads and can
  // have those loads in flight while it searches.  The first two draws are kept apart (the
  // level-0 staging lies between them): the workgroups that start together then hold
  // interleaved chunks rather than pairs of neighbours, which keeps chunk order close to the
  // order in time that the look-back counts on.
  // With no more chunks than workgroups every workgroup's first draw is its only chunk: the
  // later draws would all come back past the end, and each costs its turn at the one counter
  // (small inputs are bound by such latencies).
  const bool single = (u64)gridDim.x * kChunk >= p.n_sub;
  if (tid == 0) s_next[0] = atomicAdd(p.ticket, (u32)kChunk);
  stage_level0(p, top, bst, n_bst, kOut);
  __syncthreads();
  if (tid == 0) s_next[1] = single ? p.n_sub : atomicAdd(p.ticket, (u32)kChunk);
  u32 base = s_next[0];
  __syncthreads();
  u32 nbase = s_next[1];

  const u64 span_lo = p.table[0].base;
  const u64 span_len = p.table[p.n_alloc - 1].base + p.table[p.n_alloc - 1].size - span_lo;
  // level-0 key shift (low byte) and bucket shift, passed along as one value
  u32 shifts = key_shift_for(span_len, p.key_bits) |
               (bucket_shift_for(span_len, key_shift_for(span_len, p.key_bits), p.bucket_log2) << 8) |
               (mostly_packed(p.cmid, (p.n_alloc + 63) / 64, true) ? kUseCmid : 0u) |
               (mostly_packed(p.cleaf, (p.n_alloc + 7) / 8, false) ? kUseCleaf : 0u);
  // Candidates need not spread over the table as its lines do (most pointers of a serving
  // process point into a few huge regions, whose lines do not pack): a wave counts the marked
  // nodes and lines its candidates meet and goes back to the 64-byte forms for good once they
  // are more than a quarter.  Either form gives the same answer.
  u32 marked = 0, searched = 0;

  // The output position of a chunk is looked up one round late: while this round's rows are
  // searched, the previous round's results wait in registers; by the time its prefix is
  // needed the chunks before it have long published their totals, so the look-back does not
  // stall on other workgroups.
  RoundResults<kGroups, kG> prev, cur;
  bool have_prev = false;
  prev.base = 0;
  prev.b = 0;
  prev.cnt_incl = 0;

  u64 w[kG][kWpl];  // the group of sub-tiles this wave works on next
#pragma unroll
  for (int r = 0; r < kG; ++r) load_words<kHalf>(p, base + wave * kG + r, span_lo, w[r]);

  u32 round = 0;
  for (; base < p.n_sub; ++round) {
    const u32 b = round & 1;
    u32 next = 0;
    if (tid == 0) next = single ? p.n_sub : atomicAdd(p.ticket, (u32)kChunk);  // round + 2's chunk, published at this round's barrier
    cur.base = base;
    cur.b = b;

    auto do_group = [&](auto group_c) {
      constexpr int g = decltype(group_c)::value;
      const u32 first_sub = base + (g * kWaves + wave) * kG;
      unsigned short* qi = qi_all + (b * kGroups + g) * kQwave;
      // ---- the candidates of the group's sub-tiles go to one queue, in word order, so that
      // the search runs in dense rounds of 64 and pays its round trips once per group
      u32 Q = 0;
#pragma unroll
      for (int r = 0; r < kG; ++r) {
        Filt t;
        filter_words<kHalf>(w[r], t, span_lo, span_len);
        if (Q + t.Q <= (u32)(kGR * 64)) enqueue<kHalf, !kOut>(w[r], t, r, 0, t.Q, Q, qw, qi);
        Q += t.Q;
        if constexpr (kOut) stash_words(qw + r * kSub, w[r]);
      }
      if constexpr (kOut) wave_lds_fence();
      {  // the next group's words (this chunk's or the next one's), in flight during the search
        const u32 nsub = g + 1 < kGroups ? first_sub + kWaves * kG : nbase + wave * kG;
#pragma unroll
        for (int r = 0; r < kG; ++r) load_words<kHalf>(p, nsub + r, span_lo, w[r]);
      }
#pragma unroll
      for (int r = 0; r < kGR; ++r) cur.reg[g][r] = kMiss;
      u64 H = 0;
      if (Q <= (u32)(kGR * 64)) {
        run_group<0, kGR, kOut>(p, top, span_lo, shifts, qw, Q, cur.reg[g], cur.off[g], H, marked, qi);
        run_group<3, kGR, kOut>(p, top, span_lo, shifts, qw, Q, cur.reg[g], cur.off[g], H, marked, qi);
        run_group<6, kGR, kOut>(p, top, span_lo, shifts, qw, Q, cur.reg[g], cur.off[g], H, marked, qi);
      } else {
        // more candidates than the registers keep results for: the hits go to the wave's
        // staging area as complete entries and are copied to their place a round later
        fdy_reloc* dst = kStaged ? stage_of<kGroups, kG>(p, b, g) : nullptr;
        for (int r = 0; r < kG; ++r) {
          u64 dw[kWpl];
          Filt t;
          load_words<kHalf>(p, first_sub + r, span_lo, dw);
          filter_words<kHalf>(dw, t, span_lo, span_len);
          u64* vals = kOut ? qw + r * kSub : qw;
          const u64 wb = (u64)(first_sub + r) * kSub;
          if constexpr (kStaged) H += dense_pass<kHalf, kOut, kOut, kDenseStage>(p, dw, t, top, span_lo, shifts, vals, qi, wb, dst + H, 0, marked);
          else H += dense_pass<kHalf, kOut, kOut, kDenseCount>(p, dw, t, top, span_lo, shifts, vals, qi, wb, nullptr, 0, marked);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      }
      if constexpr (kOut) {  // the group's words, hits rebased, to the output
        wave_lds_fence();
#pragma unroll
        for (int r = 0; r < kG; ++r) unstash_words(p, first_sub + r, qw + r * kSub);
      }
      searched += Q;
      if (marked * 4 > searched + 256) shifts &= ~(kUseCmid | kUseCleaf);
      cur.Q[g] = Q;
      cur.H[g] = (u32)H;
      if (lane == 0) s_cnt[b][g * kWaves + wave] = cur.H[g];
    };
    do_group(std::integral_constant<int, 0>{});
    if constexpr (kGroups > 1) do_group(std::integral_constant<int, 1>{});
    static_assert(kGroups <= 2, "groups are instantiated by hand");

    // ---- the previous chunk's exclusive prefix (closer wave), then the round's one barrier
    if (closer && have_prev) {
      const u32 pchunk = prev.base / kChunk;
      const u64 total = __shfl(prev.cnt_incl, 63);
      const u64 excl = chunk_exclusive_prefix(p.cstate, pchunk, p.spin_limit, p.d_status);
      if (lane == 0) {
        if (pchunk != 0) st_state(&p.cstate[pchunk], kFlagInc | ((excl + total) & kValMask));
        if (prev.base + kChunk >= p.n_sub) {  // the last chunk: the grand total
          *p.d_count = excl + total;
          if (excl + total > p.capacity) raise_status(p.d_status, FDY_ST_CAPACITY);
        }
        s_excl[b] = excl;
      }
    }
    if (tid == 0) s_next[b] = next;
    __syncthreads();  // counts, next ticket and the previous chunk's prefix are visible

    const u32 nnbase = s_next[b];  // the chunk of the round after the next

    const u64 cnt = lane < (u32)kUnits ? s_cnt[b][lane] : 0;
    cur.cnt_incl = wave_incl_scan_u64(cnt);  // lane l: hits of units 0..l
    {
      const u32 chunk = base / kChunk;
      const u64 total = __shfl(cur.cnt_incl, 63);  // all lanes take part in the shuffle
      if (closer && lane == 0) st_state(&p.cstate[chunk], (chunk == 0 ? kFlagInc : kFlagAgg) | total);
    }
    if (have_prev) write_round<kGroups, kG, kHalf, kOut, kStaged>(p, prev, s_excl[b], qi_all, top, span_lo, span_len, shifts, qw, marked);
    prev = cur;
    have_prev = true;
    base = nbase;
    nbase = nnbase;
  }

  // ---- drain: the last chunk this workgroup searched.  Its prefix goes to the slot that the
  // last round did not use: a slow wave may still be about to read that round's slot.
  if (have_prev) {
    const u32 db = round & 1;
    if (closer) {
      const u32 pchunk = prev.base / kChunk;
      const u64 total = __shfl(prev.cnt_incl, 63);
      const u64 excl = chunk_exclusive_prefix(p.cstate, pchunk, p.spin_limit, p.d_status);
      if (lane == 0) {
        if (pchunk != 0) st_state(&p.cstate[pchunk], kFlagInc | ((excl + total) & kValMask));
        if (prev.base + kChunk >= p.n_sub) {  // the last chunk: the grand total
          *p.d_count = excl + total;
          if (excl + total > p.capacity) raise_status(p.d_status, FDY_ST_CAPACITY);
        }
        s_excl[db] = excl;
      }
    }
    __syncthreads();
    // this workgroup is through with the shared state: the count goes out before the last
    // entries are written, so that its round trip runs beside those stores
    if (p.self_clean && closer) finish_and_reset(p);
    write_round<kGroups, kG, kHalf, kOut, kStaged>(p, prev, s_excl[db], qi_all, top, span_lo, span_len, shifts, qw, marked);
  } else if (p.self_clean && closer) {
    finish_and_reset(p);
  }
}

// ---- fused scan + rebase: out[j] = new_base[region] + offset for a hit, words[j] otherwise.
// One pass, no relocation table, hence no ordering between waves: every wave works through
// groups of kFusedG consecutive sub-tiles on its own (static grid stride).  It searches the
// group's candidates exactly as the scan does, but a hit's queue slot receives the rebased
// value; the lanes that loaded the words then take their candidates' final values back from
// the queue and store the whole sub-tile with the same coalesced 16-byte stores a copy would
// use (storing candidates one by one from the search lanes was measured at half the speed:
// 20 M scattered 8-byte writes into lines that had already left the L2).  out may be the
// input array itself: a wave has read a sub-tile completely before it writes any of it, and
// no other wave touches that sub-tile.
template <int N>
__device__ __forceinline__ void rebase_rounds(const ScanParams& p, const u32* top, u64 span_lo, u32 shifts,
                                              u64* qw, u32 Q, u32 r0, u64& H, u32& marked) {
  const u32 lane = lane_id();
  u64 wv[N];
  Found f[N];
  bool valid[N];
#pragma unroll
  for (int r = 0; r < N; ++r) {
    valid[r] = (r0 + r) * 64 + lane < Q;
    wv[r] = valid[r] ? qw[(r0 + r) * 64 + lane] : span_lo;
  }
  search<N, false, true>(p, top, span_lo, shifts, wv, f, marked);
  u64 nb[N];
#pragma unroll
  for (int r = 0; r < N; ++r) nb[r] = valid[r] && f[r].hit ? *f[r].nb : 0;
#pragma unroll
  for (int r = 0; r < N; ++r) {
    const bool hit = valid[r] && f[r].hit;
    if (hit) qw[(r0 + r) * 64 + lane] = nb[r] + f[r].offset;  // a miss keeps its value
    H += __popcll(ballot(hit));
  }
}

// Rebases queue entries [0, Q) in place, in rounds of 64, up to three rounds interleaved.
__device__ __forceinline__ void rebase_queue(const ScanParams& p, const u32* top, u64 span_lo, u32 shifts,
                                             u64* qw, u32 Q, u64& H, u32& marked) {
  const u32 nr = (Q + 63) >> 6;
  for (u32 r0 = 0; r0 < nr; r0 += 3) {
    const u32 left = nr - r0;
    if (left >= 3) rebase_rounds<3>(p, top, span_lo, shifts, qw, Q, r0, H, marked);
    else if (left == 2) rebase_rounds<2>(p, top, span_lo, shifts, qw, Q, r0, H, marked);
    else rebase_rounds<1>(p, top, span_lo, shifts, qw, Q, r0, H, marked);
  }
}

// Candidates with rank in [win, win + wn) take their final value back from queue slots
// qoff + [0, wn).
__device__ __forceinline__ void dequeue(u64 (&w)[kWpl], const Filt& t, u32 win, u32 wn, u32 qoff,
                                        const u64* qw) {
  wave_lds_fence();
#pragma unroll
  for (int r = 0; r < kWpl; ++r)
    if (t.c[r] && t.crank[r] - win < wn) w[r] = qw[qoff + t.crank[r] - win];
  wave_lds_fence();
}

constexpr int kFusedG = 2;  // sub-tiles per group

__global__ __launch_bounds__(kBlock) void scan_rebase_kernel(ScanParams p) {
  constexpr u32 kQwave = kFusedG * kQcap;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  u32* top = reinterpret_cast<u32*>(smem_raw);
  unsigned short* bst = reinterpret_cast<unsigned short*>(top + p.top_n);
  const u32 n_bst = (1u << p.bucket_log2) + 1;
  unsigned char* qbase = smem_raw + (size_t)p.top_n * 4 + (((size_t)n_bst * 2 + 15) & ~(size_t)15);
  const u32 tid = threadIdx.x;
  const u32 lane = tid & 63;
  const u32 wave = tid >> 6;
  u64* qw = reinterpret_cast<u64*>(qbase) + wave * kQwave;
  unsigned short* qi = reinterpret_cast<unsigned short*>(qbase + (size_t)kWaves * kQwave * 8) + wave * kQwave;
  if (!prepared_ok(p)) {  // every workgroup sees the same: nothing is read or written
    if (blockIdx.x == 0 && tid == 0) raise_status(p.d_status, FDY_ST_BAD_PREPARED);
    return;
  }
  stage_level0(p, top, bst, n_bst);
  __syncthreads();

  const u64 span_lo = p.table[0].base;
  const u64 span_len = p.table[p.n_alloc - 1].base + p.table[p.n_alloc - 1].size - span_lo;
  u32 shifts = key_shift_for(span_len, p.key_bits) |
               (bucket_shift_for(span_len, key_shift_for(span_len, p.key_bits), p.bucket_log2) << 8) |
               (mostly_packed(p.cmid, (p.n_alloc + 63) / 64, true) ? kUseCmid : 0u) |
               (mostly_packed(p.cleaf, (p.n_alloc + 7) / 8, false) ? kUseCleaf : 0u);
  // Candidates need not spread over the table as its lines do (most pointers of a serving
  // process point into a few huge regions, whose lines do not pack): a wave counts the marked
  // nodes and lines its candidates meet and goes back to the 64-byte forms for good once they
  // are more than a quarter.  Either form gives the same answer.
  u32 marked = 0, searched = 0;

  // consecutive waves of a workgroup take consecutive groups; workgroups stride over the rest
  const u32 n_groups = (p.n_sub + kFusedG - 1) / kFusedG;
  const u32 stride = gridDim.x * kWaves;
  u32 grp = blockIdx.x * kWaves + wave;
  u64 H = 0;
  u64 w[kFusedG][kWpl];
  if (grp < n_groups) {
#pragma unroll
    for (int r = 0; r < kFusedG; ++r) load_words<false>(p, grp * kFusedG + r, span_lo, w[r]);
  }
  for (; grp < n_groups; grp += stride) {
    const u32 first_sub = grp * kFusedG;
    Filt t[kFusedG];
    u32 qoff[kFusedG];
    u32 Q = 0;
#pragma unroll
    for (int r = 0; r < kFusedG; ++r) {
      filter_words<false>(w[r], t[r], span_lo, span_len);
      qoff[r] = Q;
      Q += t[r].Q;
    }
    // the next group's words, in flight during the search
    const bool more = grp + stride < n_groups;
    u64 nw[kFusedG][kWpl];
    if (more) {
#pragma unroll
      for (int r = 0; r < kFusedG; ++r) load_words<false>(p, (grp + stride) * kFusedG + r, span_lo, nw[r]);
    }
    if (Q <= kQwave) {
#pragma unroll
      for (int r = 0; r < kFusedG; ++r) enqueue<false>(w[r], t[r], r, 0, t[r].Q, qoff[r], qw, qi);
      rebase_queue(p, top, span_lo, shifts, qw, Q, H, marked);
#pragma unroll
      for (int r = 0; r < kFusedG; ++r) dequeue(w[r], t[r], 0, t[r].Q, qoff[r], qw);
    } else {
      // dense group: sub-tile by sub-tile (instantiated, not looped: the words stay in
      // registers), in windows of the queue's size
      auto dense_row = [&](auto row_c) {
        constexpr int r = decltype(row_c)::value;
        for (u32 win = 0; win < t[r].Q; win += kQwave) {
          const u32 wn = t[r].Q - win < kQwave ? t[r].Q - win : kQwave;
          enqueue<false>(w[r], t[r], 0, win, wn, 0, qw, qi);
          rebase_queue(p, top, span_lo, shifts, qw, wn, H, marked);
          dequeue(w[r], t[r], win, wn, 0, qw);
        }
      };
      dense_row(std::integral_constant<int, 0>{});
      dense_row(std::integral_constant<int, 1>{});
      static_assert(kFusedG == 2, "rows are instantiated by hand");
    }
    searched += Q;
    if (marked * 4 > searched + 256) shifts &= ~(kUseCmid | kUseCleaf);
#pragma unroll
    for (int r = 0; r < kFusedG; ++r) store_words<true>(p, first_sub + r, w[r]);
    if (more) {
#pragma unroll
      for (int r = 0; r < kFusedG; ++r)
#pragma unroll
        for (int k = 0; k < kWpl; ++k) w[r][k] = nw[r][k];
    }
  }
  // The count: every wave adds its hits to the accumulator in the scan's state; the last
  // workgroup to finish publishes the sum and leaves the state zeroed for the next call.
  __shared__ u32 s_last;
  if (lane == 0 && H)
    __hip_atomic_fetch_add(p.acc, H, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the addition has been performed
  __syncthreads();
  if (tid == 0) s_last = __hip_atomic_fetch_add(p.done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == gridDim.x;
  __syncthreads();
  if (s_last && tid == 0) {
    *p.d_count = __hip_atomic_load(p.acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p.acc, (u64)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p.done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

struct ScanInit {
  const fdy_alloc* table;
  u32 n_alloc;
  u32 build;  // 0: only the state is cleared (the table's hierarchy exists already)
  u32 top_n;
  u32 sampled;  // level-0 keys that are real (the rest is padding)
  // level 0 in its two forms: keys of 32 bits with up to 2^14 buckets, keys of 16 bits with up
  // to 2^13 (see key_shift_for)
  u32* top;
  unsigned short* bstart;
  u32 bucket_log2;
  unsigned short* top16;
  unsigned short* bstart16;
  u32 bucket16_log2;
  u32 levels;
  u32 f0_log2;
  u64* mid[kMaxMid];
  u32 mid_len[kMaxMid];
  uint4* leaf;     // packed table lines, or null
  u32 leaf_lines;  // ceil(n_alloc / 8) when built
  uint4* cleaf;    // compact table lines (as many), or null
  uint4* cmid;     // compact nodes of packed level 1, or null
  u32 cmid_nodes;  // ceil(n_alloc / 64) when built
  u64* cstate;   // state to clear (null: none)
  u32 n_chunks;
  u32* header;   // the 64 counters in front of the chunk states
  u64* d_count;  // written 0 if not null (calls that find nothing to launch)
  u64* prepared;  // a prepared table's first block: 32 words, the first four from hdr, the rest 0
  PreparedHeader hdr;
};

// Line i of the compact table copy together with the new bases of its eight regions, in one
// 128-byte memory line (32 bytes of it unused): built per call of the ordered scan with output,
// from that call's base map.
// One thread per 16-byte piece, so that reads and writes are whole lines.
__global__ void scan_leafmap_kernel(const uint4* cleaf, const u64* new_base, u32 n_alloc, u32 lines, uint4* out) {
  const u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  const u64 i = t >> 3;
  const u32 piece = (u32)t & 7;
  if (i >= lines || piece >= 6) return;
  uint4 v;
  if (piece < 2) {
    v = cleaf[i * 2 + piece];
  } else {
    const u64 r = i * 8 + (piece - 2) * 2;  // this piece's two regions
    const u64 a = r < n_alloc ? new_base[r] : 0, b = r + 1 < n_alloc ? new_base[r + 1] : 0;
    v = make_uint4((u32)a, (u32)(a >> 32), (u32)b, (u32)(b >> 32));
  }
  out[t] = v;
}

// Builds the level-0 keys and the packed mid levels, clears the chunk states and counters.
__global__ void scan_init_kernel(ScanInit a) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (a.cstate && i < a.n_chunks) a.cstate[i] = 0;
  if (a.header && i < 64) a.header[i] = 0;
  if (a.d_count && i == 0) *a.d_count = 0;
  if (a.prepared && i < 32) {
    const u64 h[4] = {a.hdr.magic, (u64)a.hdr.n_alloc | ((u64)a.hdr.top_log2 << 32), a.hdr.max_words, a.hdr.table_ptr};
    a.prepared[i] = i < 4 ? h[i] : 0;
  }
  if (!a.build) return;
  const u64 span_lo = a.n_alloc ? a.table[0].base : 0;
  const u64 span_len =
      a.n_alloc ? a.table[a.n_alloc - 1].base + a.table[a.n_alloc - 1].size - span_lo : 1;
  const u32 sh0 = 3 * a.levels + a.f0_log2;
  {
    const u32 key_shift = key_shift_for(span_len, 31);
    if (i < a.top_n) {
      const u64 j = i << sh0;
      a.top[i] = j < a.n_alloc ? (u32)((a.table[j].base - span_lo) >> key_shift) : 0xffffffffu;
    }
    if (i <= (1ull << a.bucket_log2)) {
      // bucket i starts at key value i << shift: how many level-0 keys lie below it
      const u64 target = i << bucket_shift_for(span_len, key_shift, a.bucket_log2);
      u32 lo = 0, hi = a.sampled;
      while (lo < hi) {
        const u32 mid = lo + ((hi - lo) >> 1);
        if (((a.table[(u64)mid << sh0].base - span_lo) >> key_shift) < target) lo = mid + 1;
        else hi = mid;
      }
      a.bstart[i] = (unsigned short)lo;
    }
  }
  {
    const u32 key_shift = key_shift_for(span_len, 16 + a.bucket16_log2);
    if (i < a.top_n) {
      const u64 j = i << sh0;
      a.top16[i] = j < a.n_alloc ? (unsigned short)((a.table[j].base - span_lo) >> key_shift) : (unsigned short)0xffffu;
    }
    if (i <= (1ull << a.bucket16_log2)) {
      const u64 target = i << bucket_shift_for(span_len, key_shift, a.bucket16_log2);
      u32 lo = 0, hi = a.sampled;
      while (lo < hi) {
        const u32 mid = lo + ((hi - lo) >> 1);
        if (((a.table[(u64)mid << sh0].base - span_lo) >> key_shift) < target) lo = mid + 1;
        else hi = mid;
      }
      a.bstart16[i] = (unsigned short)lo;
    }
  }
  for (u32 lv = 1; lv <= a.levels; ++lv) {
    if (i < a.mid_len[lv - 1]) {
      const u64 j = i << (3 * lv);
      a.mid[lv - 1][i] = j < a.n_alloc ? a.table[j].base : ~0ull;
    }
  }
  if (i < a.leaf_lines) {
    // line i of the packed table: {(base - base of the line's first entry) >> s, size >> s} per
    // entry in 32 bits each, s the largest shift that loses no bit of any of the sixteen values
    // (allocators hand out aligned blocks, so s is usually 9 or more and regions far beyond
    // 4 GiB still pack).  The first entry's distance is 0 by definition; its slot holds s.
    // First word 0xffffffff: "read this line from the table" (a value does not fit even
    // shifted, or the line is the last, partial one).
    // The compact form of the same line: {distance >> sd : 12 bits, size >> ss : 20 bits} per
    // entry in one 32-bit word, sd and ss the trailing zeros common to the distances and to the
    // sizes, kept in the first entry's distance bits (sd low).  First word 0xffffffff (no
    // packed line has it: sd = ss = 63 leaves no size of 20 set bits): "read the 64-byte line".
    const u64 e0 = i * 8;
    u32 d[8] = {0, 0, 0, 0, 0, 0, 0, 0}, z[8] = {0, 0, 0, 0, 0, 0, 0, 0}, cw[8];
    bool fits = e0 + 8 <= a.n_alloc, cfits = fits;
    u32 sh = 0;
    if (fits) {
      const u64 b0 = a.table[e0].base;
      u64 dh[8], zh[8], any_d = 0, any_z = 0;
#pragma unroll
      for (int h = 0; h < 8; ++h) {
        dh[h] = a.table[e0 + h].base - b0;
        zh[h] = a.table[e0 + h].size;
        any_d |= dh[h];
        any_z |= zh[h];
      }
      const u64 any = any_d | any_z;
      sh = any ? (u32)__ffsll((long long)any) - 1u : 0u;  // trailing zeros common to all values
      if (sh > 31u) sh = 31u;
      const u32 sd = any_d ? (u32)__ffsll((long long)any_d) - 1u : 0u;
      const u32 ss = any_z ? (u32)__ffsll((long long)any_z) - 1u : 0u;
#pragma unroll
      for (int h = 0; h < 8; ++h) {
        fits = fits && ((dh[h] >> sh) >> 32) == 0 && ((zh[h] >> sh) >> 32) == 0;
        d[h] = (u32)(dh[h] >> sh);
        z[h] = (u32)(zh[h] >> sh);
        cfits = cfits && ((dh[h] >> sd) >> 12) == 0 && ((zh[h] >> ss) >> 20) == 0;
        cw[h] = ((u32)(dh[h] >> sd) << 20) | ((u32)(zh[h] >> ss) & 0xfffffu);
      }
      d[0] = sh;
      cw[0] |= (sd | (ss << 6)) << 20;
    }
#pragma unroll
    for (int h = 0; h < 4; ++h)
      a.leaf[i * 4 + h] = fits ? make_uint4(d[2 * h], z[2 * h], d[2 * h + 1], z[2 * h + 1])
                               : make_uint4(0xffffffffu, 0, 0xffffffffu, 0);
    if (a.cleaf) {
#pragma unroll
      for (int h = 0; h < 2; ++h)
        a.cleaf[i * 2 + h] = cfits ? make_uint4(cw[4 * h], cw[4 * h + 1], cw[4 * h + 2], cw[4 * h + 3])
                                   : make_uint4(0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu);
    }
  }
  if (i < a.cmid_nodes) {
    // node i of packed level 1 (every 8th base, 8 keys) in 32 bytes: {key 0; f1 f2 f3; f4 f5 f6;
    // f7 s}, f_h = (key h - key 0) >> s in 21 bits each, s the trailing zeros common to the
    // seven distances.  Last word ~0: "read the 64-byte node" (a distance does not fit, or the
    // node has padding keys).
    const u64 k0 = i * 64;
    bool fits = k0 + 56 < a.n_alloc;
    u64 f[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    u64 b0 = 0;
    u32 sh = 0;
    if (fits) {
      b0 = a.table[k0].base;
      u64 any = 0;
#pragma unroll
      for (int h = 1; h < 8; ++h) {
        f[h] = a.table[k0 + 8 * h].base - b0;
        any |= f[h];
      }
      sh = any ? (u32)__ffsll((long long)any) - 1u : 0u;
#pragma unroll
      for (int h = 1; h < 8; ++h) {
        f[h] >>= sh;
        fits = fits && (f[h] >> 21) == 0;
      }
    }
    const u64 a1 = f[1] | (f[2] << 21) | (f[3] << 42), a2 = f[4] | (f[5] << 21) | (f[6] << 42);
    const u64 a3 = fits ? (f[7] | ((u64)sh << 21)) : ~0ull;
    a.cmid[i * 2] = make_uint4((u32)b0, (u32)(b0 >> 32), (u32)a1, (u32)(a1 >> 32));
    a.cmid[i * 2 + 1] = make_uint4((u32)a2, (u32)(a2 >> 32), (u32)a3, (u32)(a3 >> 32));
  }
}

// (a2) one wave per boundary: lower bound of word_off[s] among the reloc words.
__global__ void reloc_segment_kernel(const fdy_reloc* relocs, const u64* d_count, u64 capacity,
                                     const u64* word_off, u32 n_off, u64* reloc_off) {
  const u32 s = blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6);
  if (s >= n_off) return;
  u64 n = *d_count;
  if (n > capacity) n = capacity;
  const u64 target = word_off[s];
  const u32 r = wave_lower_bound([&](u32 i) { return (u64)relocs[i].word; }, 0u, (u32)n, target);
  if (lane_id() == 0) reloc_off[s] = r;
}

u32 pow2_ceil(u32 v) {
  u32 p = 1;
  while (p < v) p <<= 1;
  return p;
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// The search hierarchy of one table, as it lies in memory (a caller's prepared buffer or the
// front of a workspace).  Offsets are relative to the block's start.
struct TablePlan {
  u32 top_n, levels, f0_log2, sampled, bucket_log2, bucket16_log2;
  u32 mid_len[kMaxMid];
  u32 leaf_lines, cmid_nodes;
  size_t off_top, off_bst, off_top16, off_bst16, off_mid[kMaxMid], off_leaf, off_cleaf, off_cmid, off_leafmap, bytes;
};

bool plan_table(u32 n_alloc, TablePlan* pl) {
  const u32 top_cap = 1u << fdy__tune_get(FDY_TUNE_SCAN_TOP_LOG2);
  // smallest sampling stride 2^f0_log2 * 8^levels (levels >= 2 unless the whole table fits)
  // for which the sampled bases fit the LDS level
  u32 levels = 0, f0_log2 = 0;
  auto sampled_at = [&](u32 lv, u32 f) { return (u32)(((u64)n_alloc + (1ull << (3 * lv + f)) - 1) >> (3 * lv + f)); };
  if (n_alloc > top_cap) {
    // at least two levels below the LDS level: a single one would read its table lines with
    // dependent probes (they have no packed copy, which takes the exact first base that the
    // level above the lines supplies), and that is slower than one more whole-node fetch
    levels = 2;
    while (sampled_at(levels, f0_log2) > top_cap) {
      if (++f0_log2 == 3) {
        f0_log2 = 0;
        ++levels;
      }
    }
  }
  if (levels > (u32)kMaxMid) return false;
  const u32 sampled = sampled_at(levels, f0_log2);
  pl->top_n = pow2_ceil(sampled < 2 ? 2 : sampled);
  pl->levels = levels;
  pl->f0_log2 = f0_log2;
  pl->sampled = sampled;
  size_t off = 0;
  // level 0, 32-bit keys: one bucket per key, at most 2^14 (16-bit starts, 32 KiB of LDS)
  pl->off_top = off;
  off += align256((size_t)pl->top_n * 4);
  pl->bucket_log2 = 0;
  while ((2u << pl->bucket_log2) <= pl->top_n && pl->bucket_log2 < 14u) ++pl->bucket_log2;
  pl->off_bst = off;
  off += align256((((size_t)1 << pl->bucket_log2) + 1) * 2);
  // level 0, 16-bit keys (launches that need the LDS for a copy of the words): at most 2^13 buckets
  pl->off_top16 = off;
  off += align256((size_t)pl->top_n * 2);
  pl->bucket16_log2 = pl->bucket_log2 < 13u ? pl->bucket_log2 : 13u;
  pl->off_bst16 = off;
  off += align256((((size_t)1 << pl->bucket16_log2) + 1) * 2);
  for (int j = 0; j < kMaxMid; ++j) {
    pl->mid_len[j] = 0;
    pl->off_mid[j] = off;
  }
  // packed level lv holds every 8^lv-th base.  Below the top it is read in nodes of 8 keys
  // (one per parent); the level right under level 0 exists only when a level-0 key spans
  // several of its entries (f0_log2 > 0) and is read in runs of 2^f0_log2 keys.
  const u32 top_lv = f0_log2 ? levels : (levels ? levels - 1 : 0);
  for (u32 lv = 1; lv <= top_lv; ++lv) {
    u64 len;
    if (lv == levels) len = (u64)sampled << f0_log2;
    else len = (((u64)n_alloc + (1ull << (3 * (lv + 1))) - 1) >> (3 * (lv + 1))) * 8;
    pl->mid_len[lv - 1] = (u32)len;
    pl->off_mid[lv - 1] = off;
    off += align256((size_t)len * 8);
  }
  // the packed copy of the table pays once the table itself no longer stays in L2; it needs
  // the exact base of each line's first entry, which packed level 1 supplies
  pl->leaf_lines = (levels >= 2 && pl->mid_len[0]) ? (n_alloc + 7) / 8 : 0;
  pl->off_leaf = off;
  off += align256((size_t)pl->leaf_lines * 64);
  // the compact copies of the table and of packed level 1 (32 bytes per line / node)
  pl->cmid_nodes = pl->leaf_lines ? (n_alloc + 63) / 64 : 0;
  pl->off_cleaf = off;
  off += align256((size_t)pl->leaf_lines * 32);
  pl->off_cmid = off;
  off += align256((size_t)pl->cmid_nodes * 32);
  // the compact lines with a call's base map beside them (written by every ordered scan with output)
  pl->off_leafmap = off;
  off += align256((size_t)pl->leaf_lines * 128);
  pl->bytes = off;
  return true;
}

// What depends on the number of words: chunking, and the state that a launch counts in
// (64 counters of 32 bits, then one state word per chunk; sized for the small chunks, which
// are the more numerous).
struct RunPlan {
  u32 n_sub, groups, g, n_chunks, stage_wgs;
  size_t stage_bytes;
};

constexpr size_t kStateHeader = 256;
size_t state_bytes(u64 n_words) {
  const u64 n_sub = (n_words + kSub - 1) / kSub;
  const u64 small_chunk = (u64)kWaves * kGroupsSmall * kGSmall;
  return kStateHeader + align256((size_t)((n_sub + small_chunk - 1) / small_chunk) * 8);
}

void plan_run(u64 n_words, RunPlan* rp) {
  rp->n_sub = (u32)((n_words + kSub - 1) / kSub);
  // measured crossover: from 4,096 sub-tiles (2 Mi words) on the large chunks win even though
  // they leave compute units without a chunk; below, more and smaller chunks do
  const bool small = rp->n_sub < (1u << fdy__tune_get(FDY_TUNE_SCAN_SMALL_LOG2));
  rp->groups = small ? kGroupsSmall : kGroupsBig;
  rp->g = small ? kGSmall : kGBig;
  const u32 chunk = kWaves * rp->groups * rp->g;
  rp->n_chunks = (rp->n_sub + chunk - 1) / chunk;
  // staging for the entries of dense groups: per workgroup two chunks' worth (the chunk being
  // searched and the one waiting for its position), one entry per word
  rp->stage_wgs = rp->n_chunks < kStageWgs ? rp->n_chunks : kStageWgs;
  rp->stage_bytes = align256((size_t)rp->stage_wgs * 2 * chunk * kSub * sizeof(fdy_reloc));
}


void fill_init(ScanInit* a, const fdy_alloc* d_table, u32 n_alloc, const TablePlan& tp, unsigned char* tb) {
  a->table = d_table;
  a->n_alloc = n_alloc;
  a->build = 1;
  a->top_n = tp.top_n;
  a->sampled = tp.sampled;
  a->top = (u32*)(tb + tp.off_top);
  a->bstart = (unsigned short*)(tb + tp.off_bst);
  a->bucket_log2 = tp.bucket_log2;
  a->top16 = (unsigned short*)(tb + tp.off_top16);
  a->bstart16 = (unsigned short*)(tb + tp.off_bst16);
  a->bucket16_log2 = tp.bucket16_log2;
  a->levels = tp.levels;
  a->f0_log2 = tp.f0_log2;
  for (int j = 0; j < kMaxMid; ++j) {
    a->mid[j] = (u64*)(tb + tp.off_mid[j]);
    a->mid_len[j] = tp.mid_len[j];
  }
  a->leaf = tp.leaf_lines ? (uint4*)(tb + tp.off_leaf) : nullptr;
  a->leaf_lines = tp.leaf_lines;
  a->cleaf = tp.leaf_lines ? (uint4*)(tb + tp.off_cleaf) : nullptr;
  a->cmid = tp.cmid_nodes ? (uint4*)(tb + tp.off_cmid) : nullptr;
  a->cmid_nodes = tp.cmid_nodes;
  a->cstate = nullptr;
  a->n_chunks = 0;
  a->header = nullptr;
  a->d_count = nullptr;
  a->prepared = nullptr;
  a->hdr = PreparedHeader{};
}

u32 init_threads(const TablePlan& tp, u32 n_chunks) {
  u32 n = tp.top_n > n_chunks ? tp.top_n : n_chunks;
  for (int j = 0; j < kMaxMid; ++j)
    if (tp.mid_len[j] > n) n = tp.mid_len[j];
  if (tp.leaf_lines > n) n = tp.leaf_lines;
  if ((1u << tp.bucket_log2) + 1 > n) n = (1u << tp.bucket_log2) + 1;
  return n < 64 ? 64 : n;
}

}  // namespace
}  // namespace fdy

using namespace fdy;

extern "C" size_t fdy_scan_workspace_bytes(uint64_t n_words, uint32_t n_alloc) {
  if (n_words > kMaxWords) return 0;
  TablePlan tp;
  if (!plan_table(n_alloc, &tp)) return 0;
  return state_bytes(n_words) + tp.bytes;
}

extern "C" size_t fdy_scan_staging_bytes(uint64_t n_words) {
  if (n_words > kMaxWords) return 0;
  RunPlan rp;
  plan_run(n_words, &rp);
  return rp.stage_bytes;
}

extern "C" size_t fdy_scan_table_bytes(uint32_t n_alloc, uint64_t max_words) {
  if (max_words > kMaxWords) return 0;
  TablePlan tp;
  if (!plan_table(n_alloc, &tp)) return 0;
  return kPreparedHeader + state_bytes(max_words) + tp.bytes;
}

extern "C" int fdy_scan_table_prepare(const fdy_alloc* d_table, uint32_t n_alloc, uint64_t max_words,
                                      void* d_prepared, size_t prepared_bytes, void* hip_stream) {
  if (max_words > kMaxWords) return FDY_ERR_INVALID_ARG;
  if (n_alloc && (!d_table || ((uintptr_t)d_table & 15))) return FDY_ERR_INVALID_ARG;
  TablePlan tp;
  if (!plan_table(n_alloc, &tp)) return FDY_ERR_INVALID_ARG;
  const size_t need = kPreparedHeader + state_bytes(max_words) + tp.bytes;
  if (!d_prepared || ((uintptr_t)d_prepared & 255) || prepared_bytes < need) return FDY_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  unsigned char* pb = (unsigned char*)d_prepared;
  ScanInit a;
  fill_init(&a, d_table, n_alloc, tp, pb + kPreparedHeader);
  a.prepared = (u64*)pb;
  a.hdr.magic = kPreparedMagic;
  a.hdr.n_alloc = n_alloc;
  a.hdr.top_log2 = (u32)fdy__tune_get(FDY_TUNE_SCAN_TOP_LOG2);
  a.hdr.max_words = max_words;
  a.hdr.table_ptr = (u64)(uintptr_t)d_table;
  a.header = (u32*)(pb + kPreparedHeader + tp.bytes);
  a.cstate = (u64*)(pb + kPreparedHeader + tp.bytes + kStateHeader);
  a.n_chunks = (u32)((state_bytes(max_words) - kStateHeader) / 8);
  a.d_count = nullptr;
  const u32 n_init = init_threads(tp, a.n_chunks);
  launch(FDY_PROF_SCAN_INIT, scan_init_kernel, dim3((n_init + 255) / 256), dim3(256), 0, stream, a);
  FDY_HIP_TRY(hipGetLastError());
  return FDY_OK;
}

// Shared by the scans: checks, where hierarchy and state lie (in the caller's prepared table, or
// built into the workspace by a launch of this call), then the main kernel.
static int scan_launch(const uint64_t* d_words, uint64_t n_words, const fdy_alloc* d_table,
                       uint32_t n_alloc, fdy_reloc* d_relocs, uint64_t reloc_capacity, uint64_t* d_count,
                       const uint64_t* d_new_base, uint64_t* d_out, const void* d_prepared, void* d_workspace,
                       size_t workspace_bytes, uint32_t* d_status, void* hip_stream, bool half = false,
                       bool ordered_out = false) {
  const bool fused = d_out != nullptr && !ordered_out;  // no relocation table, no ordering
  if (n_words > kMaxWords) return FDY_ERR_INVALID_ARG;
  if (!d_count) return FDY_ERR_INVALID_ARG;
  if (n_words && (!d_words || ((uintptr_t)d_words & 15))) return FDY_ERR_INVALID_ARG;
  if (n_alloc && (!d_table || ((uintptr_t)d_table & 15))) return FDY_ERR_INVALID_ARG;
  if (reloc_capacity && (!d_relocs || ((uintptr_t)d_relocs & 15))) return FDY_ERR_INVALID_ARG;
  if (d_prepared && ((uintptr_t)d_prepared & 255)) return FDY_ERR_INVALID_ARG;
  TablePlan tp;
  if (!plan_table(n_alloc, &tp)) return FDY_ERR_INVALID_ARG;
  RunPlan rp;
  plan_run(n_words, &rp);
  // where things lie
  unsigned char* ws = (unsigned char*)d_workspace;
  unsigned char *state, *tb, *stage;
  if (d_prepared) {
    // the caller vouches for the buffer (made by fdy_scan_table_prepare for this table and at
    // least this many words, under the same tuning); only the staging comes from the workspace
    unsigned char* pb = (unsigned char*)const_cast<void*>(d_prepared);
    tb = pb + kPreparedHeader;
    state = tb + tp.bytes;
    if (ws && ((uintptr_t)ws & 255)) return FDY_ERR_WORKSPACE;
    stage = ws && workspace_bytes >= rp.stage_bytes ? ws : nullptr;
  } else {
    const size_t need = state_bytes(n_words) + tp.bytes;
    if (!ws || ((uintptr_t)ws & 255) || workspace_bytes < need) return FDY_ERR_WORKSPACE;
    state = ws;
    tb = ws + state_bytes(n_words);
    stage = workspace_bytes >= need + rp.stage_bytes ? tb + tp.bytes : nullptr;
  }
  hipStream_t stream = (hipStream_t)hip_stream;
  (void)hipGetLastError();  // drop any stale error left by earlier, unrelated runtime calls
  int dev = 0, n_cu = 256;
  FDY_HIP_TRY(hipGetDevice(&dev));
  FDY_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  const u32 per_cu = (u32)fdy__tune_get(FDY_TUNE_SCAN_WG_PER_CU);
  u32 grid = (u32)n_cu * per_cu;  // persistent workgroups
  if (grid > rp.n_chunks) grid = rp.n_chunks;
  if (grid > rp.stage_wgs) grid = rp.stage_wgs;  // kStageWgs bounds every launch: the staging is sized for it
  const bool nothing = rp.n_sub == 0 || n_alloc == 0;  // no word can be a pointer
  ScanInit a;
  fill_init(&a, d_table, n_alloc, tp, tb);
  if (d_prepared) {
    if (nothing) {  // only the count is owed
      ScanInit z = ScanInit{};
      z.d_count = (u64*)d_count;
      hipLaunchKernelGGL(scan_init_kernel, dim3(1), dim3(64), 0, stream, z);
      FDY_HIP_TRY(hipGetLastError());
    }
  } else {
    a.header = (u32*)state;
    a.cstate = (u64*)(state + kStateHeader);
    a.n_chunks = rp.n_chunks;
    a.d_count = nothing ? (u64*)d_count : nullptr;
    const u32 n_init = init_threads(tp, rp.n_chunks);
    launch(FDY_PROF_SCAN_INIT, scan_init_kernel, dim3((n_init + 255) / 256), dim3(256), 0, stream, a);
    FDY_HIP_TRY(hipGetLastError());
  }
  if (rp.n_sub == 0) return FDY_OK;
  if (n_alloc == 0) {  // nothing can be a pointer; forms with an output still owe the copy
    if (d_out && d_out != d_words)
      FDY_HIP_TRY(hipMemcpyAsync(d_out, d_words, n_words * 8, hipMemcpyDeviceToDevice, stream));
    return FDY_OK;
  }
  
  ScanParams p;
  p.words = (const u64*)d_words;
  p.n_words = n_words;
  p.table = d_table;
  p.n_alloc = n_alloc;
  p.relocs = d_relocs;
  p.capacity = reloc_capacity;
  p.d_count = (u64*)d_count;
  // state: counter 0 = ticket, 1 = finished workgroups, 2..3 = hit accumulator (64 bits)
  p.ticket = (u32*)state;
  p.done = (u32*)state + 1;
  p.acc = (u64*)state + 1;
  p.cstate = (u64*)(state + kStateHeader);
  p.n_chunks = rp.n_chunks;
  p.self_clean = d_prepared ? 1u : 0u;
  p.prepared = (const u64*)d_prepared;
  p.top_log2 = (u32)fdy__tune_get(FDY_TUNE_SCAN_TOP_LOG2);
  // level 0 in the form this launch stages in LDS
  p.top = ordered_out ? (const u32*)a.top16 : a.top;
  p.bstart = ordered_out ? a.bstart16 : a.bstart;
  p.bucket_log2 = ordered_out ? a.bucket16_log2 : a.bucket_log2;
  p.key_bits = ordered_out ? 16 + a.bucket16_log2 : 31;
  for (int j = 0; j < kMaxMid; ++j) p.mid[j] = a.mid[j];
  p.leaf = a.leaf;
  p.cmid = a.cmid;
  p.cleaf = a.cleaf;
  p.leafmap = nullptr;
  if ((ordered_out || fused) && tp.leaf_lines) {
    uint4* lm = (uint4*)(tb + tp.off_leafmap);
    launch(FDY_PROF_SCAN_RECORDS, scan_leafmap_kernel, dim3((u32)(((u64)tp.leaf_lines * 8 + 255) / 256)), dim3(256),
           0, stream, (const uint4*)a.cleaf, (const u64*)d_new_base, n_alloc, tp.leaf_lines, lm);
    FDY_HIP_TRY(hipGetLastError());
    p.leafmap = lm;
  }
  p.stage = (fdy_reloc*)stage;
  p.n_sub = rp.n_sub;
  p.top_n = tp.top_n;
  p.levels = tp.levels;
  p.f0_log2 = tp.f0_log2;
  p.d_status = d_status;
  p.spin_limit = (u32)fdy__tune_get(FDY_TUNE_SCAN_SPIN_LIMIT);
  p.new_base = (const u64*)d_new_base;
  p.out = (u64*)d_out;

  const size_t lds0 = level0_key_bytes(tp.top_n, ordered_out) + (((((size_t)1 << p.bucket_log2) + 1) * 2 + 15) & ~(size_t)15);
  if (fused) {
    const size_t lds = lds0 + (size_t)kWaves * kFusedG * kQcap * 10;
    const u32 n_groups = (rp.n_sub + kFusedG - 1) / kFusedG;
    u32 fgrid = (u32)n_cu;  // one workgroup per compute unit (256 registers per lane)
    if (fgrid > (n_groups + kWaves - 1) / kWaves) fgrid = (n_groups + kWaves - 1) / kWaves;
    FDY_HIP_TRY(hipFuncSetAttribute((const void*)scan_rebase_kernel,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    launch(FDY_PROF_SCAN_REBASE, scan_rebase_kernel, dim3(fgrid), dim3(kBlock), lds, stream, p);
    FDY_HIP_TRY(hipGetLastError());
    return FDY_OK;
  }
  // per wave: the value queue (or, with a rebased output, the words of a group) and the
  // index queues of two chunks
  const size_t lds = lds0 + (size_t)kWaves * rp.g * ((ordered_out ? (size_t)kSub : (size_t)kQcap) * 8 +
                                                      (size_t)kQcap * 2 * 2 * rp.groups);
  auto pick = [&](auto staged_c) {
    constexpr bool st = decltype(staged_c)::value;
    return rp.g == kGSmall ? (half          ? scan_kernel<kGroupsSmall, kGSmall, true, false, st>
                              : ordered_out ? scan_kernel<kGroupsSmall, kGSmall, false, true, st>
                                            : scan_kernel<kGroupsSmall, kGSmall, false, false, st>)
                           : (half          ? scan_kernel<kGroupsBig, kGBig, true, false, st>
                              : ordered_out ? scan_kernel<kGroupsBig, kGBig, false, true, st>
                                            : scan_kernel<kGroupsBig, kGBig, false, false, st>);
  };
  auto kern = stage ? pick(std::true_type{}) : pick(std::false_type{});
  FDY_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const int slot = ordered_out ? FDY_PROF_SCAN_OUT : FDY_PROF_SCAN_MAIN;
  launch(slot, kern, dim3(grid), dim3(kBlock), lds, stream, p);
  FDY_HIP_TRY(hipGetLastError());
  return FDY_OK;
}

extern "C" int fdy_scan_pointers(const uint64_t* d_words, uint64_t n_words, const fdy_alloc* d_table,
                                 uint32_t n_alloc, fdy_reloc* d_relocs, uint64_t reloc_capacity,
                                 uint64_t* d_count, const void* d_prepared, void* d_workspace,
                                 size_t workspace_bytes,
                                 uint32_t* d_status, void* hip_stream) {
  return scan_launch(d_words, n_words, d_table, n_alloc, d_relocs, reloc_capacity, d_count, nullptr, nullptr,
                     d_prepared, d_workspace, workspace_bytes, d_status, hip_stream);
}

extern "C" int fdy_scan_pointers_stride4(const uint32_t* d_units, uint64_t n_units, const fdy_alloc* d_table,
                                         uint32_t n_alloc, fdy_reloc* d_relocs, uint64_t reloc_capacity,
                                         uint64_t* d_count, const void* d_prepared, void* d_workspace,
                                 size_t workspace_bytes,
                                         uint32_t* d_status, void* hip_stream) {
  // position q pairs unit q with unit q + 1: one position less than units
  const uint64_t n_pos = n_units >= 2 ? n_units - 1 : 0;
  if (n_units && !d_units) return FDY_ERR_INVALID_ARG;
  return scan_launch(reinterpret_cast<const uint64_t*>(d_units), n_pos, d_table, n_alloc, d_relocs,
                     reloc_capacity, d_count, nullptr, nullptr, d_prepared, d_workspace, workspace_bytes, d_status,
                     hip_stream, true);
}

extern "C" int fdy_scan_rebase(const uint64_t* d_words, uint64_t n_words, const fdy_alloc* d_table,
                               uint32_t n_alloc, const uint64_t* d_new_base, uint64_t* d_out_words,
                               uint64_t* d_count, const void* d_prepared, void* d_workspace,
                                 size_t workspace_bytes,
                               uint32_t* d_status, void* hip_stream) {
  if (n_words && (!d_out_words || ((uintptr_t)d_out_words & 15))) return FDY_ERR_INVALID_ARG;
  if (n_alloc && (!d_new_base || ((uintptr_t)d_new_base & 7))) return FDY_ERR_INVALID_ARG;
  if (n_words == 0) {  // nothing to write; keep the count defined
    if (!d_count) return FDY_ERR_INVALID_ARG;
    return scan_launch(d_words, 0, d_table, n_alloc, nullptr, 0, d_count, nullptr, nullptr, d_prepared, d_workspace,
                       workspace_bytes, d_status, hip_stream);
  }
  if (d_out_words != d_words) {  // exactly the same array, or disjoint
    const uintptr_t a = (uintptr_t)d_words, b = (uintptr_t)d_out_words, len = (uintptr_t)n_words * 8;
    if (a < b + len && b < a + len) return FDY_ERR_INVALID_ARG;
  }
  return scan_launch(d_words, n_words, d_table, n_alloc, nullptr, 0, d_count, d_new_base, d_out_words,
                     d_prepared, d_workspace, workspace_bytes, d_status, hip_stream);
}

extern "C" int fdy_scan_pointers_rebase(const uint64_t* d_words, uint64_t n_words, const fdy_alloc* d_table,
                                        uint32_t n_alloc, fdy_reloc* d_relocs, uint64_t reloc_capacity,
                                        uint64_t* d_count, const uint64_t* d_new_base, uint64_t* d_out_words,
                                        const void* d_prepared, void* d_workspace, size_t workspace_bytes, uint32_t* d_status,
                                        void* hip_stream) {
  if (n_words && (!d_out_words || ((uintptr_t)d_out_words & 15))) return FDY_ERR_INVALID_ARG;
  if (n_alloc && (!d_new_base || ((uintptr_t)d_new_base & 7))) return FDY_ERR_INVALID_ARG;
  if (n_words) {  // the output is written while other workgroups still read the input
    const uintptr_t a = (uintptr_t)d_words, b = (uintptr_t)d_out_words, len = (uintptr_t)n_words * 8;
    if (a < b + len && b < a + len) return FDY_ERR_INVALID_ARG;
  }
  return scan_launch(d_words, n_words, d_table, n_alloc, d_relocs, reloc_capacity, d_count, d_new_base,
                     n_words ? d_out_words : nullptr, d_prepared, d_workspace, workspace_bytes, d_status, hip_stream, false,
                     true);
}

extern "C" int fdy_reloc_segment(const fdy_reloc* d_relocs, const uint64_t* d_count,
                                 uint64_t reloc_capacity, const uint64_t* d_word_off, uint32_t n_off,
                                 uint64_t* d_reloc_off, void* hip_stream) {
  if (n_off == 0) return FDY_OK;
  if (!d_count || !d_word_off || !d_reloc_off) return FDY_ERR_INVALID_ARG;
  if (reloc_capacity && !d_relocs) return FDY_ERR_INVALID_ARG;
  (void)hipGetLastError();
  launch(FDY_PROF_SEGMENT, reloc_segment_kernel, dim3((n_off + 3) / 4), dim3(256), 0, (hipStream_t)hip_stream,
         d_relocs, (const u64*)d_count, reloc_capacity, (const u64*)d_word_off, n_off, (u64*)d_reloc_off);
  FDY_HIP_TRY(hipGetLastError());
  return FDY_OK;
}
