"""Seeded synthetic capture archives.

These stand in for real captured-graph archives (Section 6.1 of the paper captures one
graph per batch size for 36- and 94-layer models; Appendix B shows an argument buffer of
1720 bytes mixing small integers, packed constants and opaque data).  The generator only
*plants* data and records where it planted it; it evaluates none of the method's steps
(no interval search, no hashing, no rebasing of blobs).  The planted positions are the
ground truth the oracle is pinned against.

Five named configurations exist (``make_config(1..5)``); every size can be overridden so
that CPU tests can run reduced versions with the same structure.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import layout as L

SEED0 = 0x260406664000
OLD_BASE0 = 0x7F0000000000
MiB = 1 << 20
ALIGN = 2 * MiB
U64 = np.uint64


@dataclass
class Archive:
    name: str
    table: np.ndarray  # ALLOC[A]
    words: np.ndarray  # u64[W], all graphs' argument blobs concatenated
    word_off: np.ndarray  # u64[G+1]
    nodes: np.ndarray  # NODE[sum nodes]
    node_off: np.ndarray  # u64[G+1]
    # ground truth of what was planted
    ptr_word: np.ndarray  # i64[K] ascending word indices holding planted pointers
    ptr_region: np.ndarray  # u32[K]
    ptr_offset: np.ndarray  # u64[K]
    decoy_word: np.ndarray  # i64[D] word indices holding base-1 / base+size decoys
    # templating ground truth (by construction, not by hashing)
    fp_mask: int
    graph_tmpl: np.ndarray  # u32[G]
    tmpl_graph: np.ndarray  # u32[T]
    ovr: np.ndarray  # OVR32[...]
    ovr_off: np.ndarray  # u64[G+1]
    govr: np.ndarray  # GRID_OVR[...]
    govr_off: np.ndarray  # u64[G+1]
    new_base: np.ndarray  # u64[M][A]
    map_rank: np.ndarray | None  # u32[M]
    n_ranks: int
    patch: np.ndarray  # PATCH[...]
    patch_off: np.ndarray  # u64[T*R+1]
    batch_sizes: list = field(default_factory=list)

    @property
    def n_graphs(self):
        return len(self.word_off) - 1

    @property
    def n_templates(self):
        return len(self.tmpl_graph)

    @property
    def n_maps(self):
        return self.new_base.shape[0]

    @property
    def n_alloc(self):
        return len(self.table)


# ------------------------------------------------------------------------------------
# allocation tables and base maps
# ------------------------------------------------------------------------------------
def make_table(rng, n_alloc, size_lo, size_hi, base0=OLD_BASE0, kind="granule"):
    """Deterministic-layout style table: ascending from base0, 2 MiB aligned bases,
    sizes log-uniform in [size_lo, size_hi] rounded up to 512 B, and always a gap of at
    least 2 MiB - (size mod 2 MiB) > 0 bytes after each allocation, so that base-1 and
    base+size lie in no allocation.
    kind "huge": the same with every 100th region 8 GiB (weights, KV cache).
    kind "bytes": a caching allocator's blocks instead: byte-granular sizes, 16-byte aligned
    bases, gaps of 16..1008 bytes."""
    size = np.exp(rng.uniform(np.log(size_lo), np.log(size_hi), n_alloc))
    if kind == "bytes":
        size = np.clip(size.astype(np.uint64), size_lo, size_hi).astype(np.uint64)
        step = (size + U64(15)) // U64(16) * U64(16) + rng.integers(1, 64, n_alloc).astype(np.uint64) * U64(16)
        base = np.empty(n_alloc, np.uint64)
        base[0] = base0
        if n_alloc > 1:
            base[1:] = U64(base0) + np.cumsum(step[:-1], dtype=np.uint64)
        t = np.empty(n_alloc, L.ALLOC)
        t["base"] = base
        t["size"] = size
        return t
    size = (np.ceil(size / 512.0).astype(np.uint64) * U64(512)).astype(np.uint64)
    size = np.clip(size, size_lo, size_hi).astype(np.uint64)
    if kind == "huge":
        size[::100] = U64(8 << 30)
    k = rng.integers(0, 4, n_alloc).astype(np.uint64)
    aligned = (size + U64(ALIGN - 1)) // U64(ALIGN) * U64(ALIGN)
    k = np.where((aligned == size) & (k == 0), U64(1), k)  # never touch the next base
    step = aligned + k * U64(ALIGN)
    base = np.empty(n_alloc, np.uint64)
    base[0] = base0
    if n_alloc > 1:
        base[1:] = U64(base0) + np.cumsum(step[:-1], dtype=np.uint64)
    t = np.empty(n_alloc, L.ALLOC)
    t["base"] = base
    t["size"] = size
    return t


def permuted_base_map(rng, table, start):
    """New placement: regions laid out contiguously (2 MiB aligned) from `start` in a random
    order.  Returns new_base[A] indexed by region."""
    n = len(table)
    perm = rng.permutation(n)
    aligned = (table["size"][perm] + U64(ALIGN - 1)) // U64(ALIGN) * U64(ALIGN) + U64(ALIGN)
    pos = np.empty(n, np.uint64)
    pos[0] = start
    if n > 1:
        pos[1:] = U64(start) + np.cumsum(aligned[:-1], dtype=np.uint64)
    nb = np.empty(n, np.uint64)
    nb[perm] = pos
    return nb


def table_span(table):
    return int(table["base"][0]), int(table["base"][-1] + table["size"][-1])


# ------------------------------------------------------------------------------------
# word filling
# ------------------------------------------------------------------------------------
def fill_words(rng, n, table, p_ptr, p_decoy, rest="mix"):
    """n words: fraction p_ptr planted pointers (base[i] + u, u < size[i], i uniform),
    fraction p_decoy boundary decoys (base[i]-1 or base[i]+size[i]), the rest either
    'mix' (small ints 0..65535 / packed fp32 pairs) or 'rand64' (uniform 64-bit values
    outside the table's span).  Returns words and the planted ground truth."""
    A = len(table)
    base, size = table["base"], table["size"]
    lo, hi = table_span(table)
    kind = rng.random(n)
    words = np.empty(n, np.uint64)
    ptr_idx = np.flatnonzero(kind < p_ptr)
    dec_idx = np.flatnonzero((kind >= p_ptr) & (kind < p_ptr + p_decoy))
    rest_idx = np.flatnonzero(kind >= p_ptr + p_decoy)
    del kind
    # planted pointers
    reg = rng.integers(0, A, len(ptr_idx))
    off = (rng.random(len(ptr_idx)) * size[reg]).astype(np.uint64)
    off = np.minimum(off, size[reg] - U64(1))
    # make sure both ends of a region occur
    if len(ptr_idx) >= 4:
        off[0] = 0
        off[1] = size[reg[1]] - U64(1)
    words[ptr_idx] = base[reg] + off
    # decoys
    dreg = rng.integers(0, A, len(dec_idx))
    which = rng.integers(0, 2, len(dec_idx)).astype(bool)
    words[dec_idx] = np.where(which, base[dreg] - U64(1), base[dreg] + size[dreg])
    # the rest
    m = len(rest_idx)
    if rest == "mix":
        small = rng.integers(0, 65536, m, dtype=np.uint64)
        f = rng.uniform(-8.0, 8.0, (m, 2)).astype(np.float32)
        pair = f.view(np.uint32).astype(np.uint64)
        packed = pair[:, 0] | (pair[:, 1] << U64(32))
        pick = rng.random(m) < 0.5
        vals = np.where(pick, small, packed)
    else:
        vals = rng.integers(0, 1 << 64, m, dtype=np.uint64)
        bad = (vals >= U64(lo)) & (vals < U64(hi))
        vals[bad] = vals[bad] ^ U64(1 << 63)  # span lies below 2^63: flips it out
    bad = (vals >= U64(lo - 1)) & (vals <= U64(hi))
    assert not bad.any(), "filler value inside the table span"
    words[rest_idx] = vals
    return words, ptr_idx, reg.astype(np.uint32), off, dec_idx


# ------------------------------------------------------------------------------------
# model-shaped archives (configs 2, 3, 5)
# ------------------------------------------------------------------------------------
def default_batch_sizes():
    return [1, 2, 4] + list(range(8, 513, 8))  # 67 graphs


def _blob_lens(rng, kpl, mean_target=160.0):
    """Per-slot argument-buffer lengths: 16..1024 B, multiples of 8, skewed log-uniform
    with mean near 160 B."""
    for _ in range(1000):
        u = rng.random(kpl)
        ln = np.round(16.0 * 64.0 ** (u**1.8) / 8.0).astype(np.int64) * 8
        ln = np.clip(ln, 16, 1024)
        if abs(ln.mean() - mean_target) < 10.0:
            return ln
    return ln


def make_model_archive(name, seed, layers, kpl, n_alloc, size_hi, batch_sizes, n_maps,
                       map_kind, comm_slots=(), n_ranks=0, size_lo=4096, p_ptr=0.25,
                       p_decoy=0.05, bucket_edges=(8, 128)):
    rng = np.random.default_rng(seed)
    table = make_table(rng, n_alloc, size_lo, size_hi)
    G = len(batch_sizes)
    N = layers * kpl
    # --- topology buckets by batch size (three by default: <= 8, <= 128, above)
    edges = sorted(bucket_edges)

    def bucket(bs):
        return int(np.searchsorted(edges, bs, side="left"))

    bs_slots = (2 % kpl, (kpl // 2 + 1) % kpl)
    slot_kid = rng.integers(1, 1 << 63, kpl, dtype=np.uint64)
    slot_len = _blob_lens(rng, kpl)
    for s in comm_slots:
        slot_len[s] = max(slot_len[s], 128)
    slot_block = rng.choice([64, 128, 256, 384, 512, 1024], kpl).astype(np.uint32)
    slot_gx = rng.integers(1, 64, kpl).astype(np.uint32)
    slot_gy = rng.integers(1, 8, kpl).astype(np.uint32)
    slot_flags = (rng.integers(0, 2, kpl).astype(np.uint32) << np.uint32(4))
    for s in comm_slots:
        slot_flags[s] |= 1
    shapes = []
    for b in range(len(edges) + 1):
        kid, ln = slot_kid.copy(), slot_len.copy()
        if b > 0:
            free = [s for s in range(kpl) if s not in comm_slots and s not in bs_slots]
            ch = rng.choice(free, size=min(3, len(free)), replace=False)
            kid[ch[:2]] = rng.integers(1, 1 << 63, len(ch[:2]), dtype=np.uint64)
            if len(ch) > 2:
                ln[ch[2]] = int(np.clip(ln[ch[2]] + 8 * min(b, 2), 16, 1024))
        shapes.append((kid, ln))

    # --- per-bucket base blob
    present = sorted({bucket(bs) for bs in batch_sizes})
    blobs = {}
    for b in present:
        kid, ln = shapes[b]
        node_len = np.tile(ln, layers)
        node_woff = np.concatenate([[0], np.cumsum(node_len // 8)]).astype(np.int64)
        nw = int(node_woff[-1])
        w, pidx, preg, poff, didx = fill_words(rng, nw, table, p_ptr, p_decoy, "mix")
        special = []  # words that must not be planted data
        bs_fields = []  # (node, word index in graph, high-half?)
        for layer in range(layers):
            for j, s in enumerate(bs_slots):
                node = layer * kpl + s
                special.append(node_woff[node] + 1)
                bs_fields.append((node, int(node_woff[node] + 1), j == 1))
        comm_nodes = []
        for layer in range(layers):
            for s in comm_slots:
                node = layer * kpl + s
                comm_nodes.append(node)
                special.extend(range(node_woff[node], node_woff[node] + 10))
        special = np.array(sorted(set(special)), np.int64)
        keep = ~np.isin(pidx, special)
        pidx, preg, poff = pidx[keep], preg[keep], poff[keep]
        didx = didx[~np.isin(didx, special)]
        # stub communication state of the single-rank capture (outside every allocation)
        for node in comm_nodes:
            o = int(node_woff[node])
            w[o] = U64(0xFD00000000000000 | node)  # handle stub
            w[o + 1] = U64(0 | (1 << 32))  # {rank 0, nranks 1}
            w[o + 2:o + 10] = U64(0xFDFD000000000000) + np.arange(8, dtype=np.uint64)
        blobs[b] = dict(words=w, node_len=node_len, node_woff=node_woff, pidx=pidx, preg=preg,
                        poff=poff, didx=didx, bs_fields=bs_fields, comm_nodes=comm_nodes)

    def bs_word(bs, high):
        return U64((bs << 32) | 7) if high else U64(bs)

    def grid_for(bs, s):
        return (np.uint32(slot_gx[s] * ((bs + 15) // 16)), slot_gy[s], np.uint32(1))

    # --- graphs
    words_l, nodes_l = [], []
    word_off, node_off = [0], [0]
    ptr_w, ptr_r, ptr_o, dec_w = [], [], [], []
    graph_tmpl = np.zeros(G, np.uint32)
    tmpl_graph, tmpl_of_bucket = [], {}
    ovr_l, ovr_off, govr_l, govr_off = [], [0], [], [0]
    for g, bs in enumerate(batch_sizes):
        b = bucket(bs)
        B = blobs[b]
        kid, ln = shapes[b]
        if b not in tmpl_of_bucket:
            tmpl_of_bucket[b] = len(tmpl_graph)
            tmpl_graph.append(g)
        graph_tmpl[g] = tmpl_of_bucket[b]
        is_template = tmpl_graph[graph_tmpl[g]] == g
        w = B["words"].copy()
        nd = np.zeros(N, L.NODE)
        nd["kernel_id"] = np.tile(kid, layers)
        nd["grid"][:, 0] = np.tile(slot_gx, layers)
        nd["grid"][:, 1] = np.tile(slot_gy, layers)
        nd["grid"][:, 2] = 1
        nd["block"][:, 0] = np.tile(slot_block, layers)
        nd["block"][:, 1] = 1
        nd["block"][:, 2] = 1
        nd["blob_len"] = B["node_len"]
        nd["flags"] = np.tile(slot_flags, layers)
        o = np.zeros(0 if is_template else len(B["bs_fields"]), L.OVR32)
        go = np.zeros(0 if is_template else len(B["bs_fields"]), L.GRID_OVR)
        for i, (node, widx, high) in enumerate(B["bs_fields"]):
            w[widx] = bs_word(bs, high)
            gr = grid_for(bs, node % kpl)
            nd["grid"][node] = gr
            if not is_template:
                o[i] = (widx * 8 + (4 if high else 0), bs)
                go[i] = (node, gr)
        base_w = word_off[-1]
        words_l.append(w)
        nodes_l.append(nd)
        word_off.append(base_w + len(w))
        node_off.append(node_off[-1] + N)
        ptr_w.append(B["pidx"] + base_w)
        ptr_r.append(B["preg"])
        ptr_o.append(B["poff"])
        dec_w.append(B["didx"] + base_w)
        ovr_l.append(o)
        govr_l.append(go)
        ovr_off.append(ovr_off[-1] + len(o))
        govr_off.append(govr_off[-1] + len(go))

    T = len(tmpl_graph)
    # --- rank patch tables, per (template, rank)
    patch_l, patch_off = [], [0]
    if n_ranks:
        for t in range(T):
            bsel = [b for b, tt in tmpl_of_bucket.items() if tt == t][0]
            B = blobs[bsel]
            for r in range(n_ranks):
                p = np.zeros(len(B["comm_nodes"]) * 10, L.PATCH)
                for i, node in enumerate(B["comm_nodes"]):
                    o = int(B["node_woff"][node])
                    p["word"][i * 10:(i + 1) * 10] = np.arange(o, o + 10)
                    vals = np.empty(10, np.uint64)
                    vals[0] = rng.integers(0, 1 << 63, dtype=np.uint64) | U64(1 << 63)
                    vals[1] = U64(r | (n_ranks << 32))
                    peer = np.arange(8, dtype=np.uint64)
                    vals[2:] = (U64(0x600000000000) + (peer << U64(36))
                                + rng.integers(0, 1 << 26, 8, dtype=np.uint64) * U64(256))
                    p["value"][i * 10:(i + 1) * 10] = vals
                patch_l.append(p)
                patch_off.append(patch_off[-1] + len(p))
    else:
        patch_off = [0] * (T * max(n_ranks, 0) + 1)

    # --- base maps
    lo, hi = table_span(table)
    assert hi - lo < (1 << 40), "old span must stay below 1 TiB for the map recipes"
    if map_kind == "permute":  # fresh instances: random region order, own 1 TiB window each
        new_base = np.stack([permuted_base_map(rng, table, 0x800000000000 + (m << 40))
                             for m in range(n_maps)])
        for m in range(n_maps):
            assert int(new_base[m].max()) + size_hi < 0x800000000000 + ((m + 1) << 40)
        map_rank = None
    elif map_kind == "rank_shift":  # simulated ranks: whole layout shifted by (m+1) TiB
        new_base = np.stack([table["base"] + U64((m + 1) << 40) for m in range(n_maps)])
        map_rank = (np.arange(n_maps) % max(n_ranks, 1)).astype(np.uint32)
    else:
        raise ValueError(map_kind)

    cat = lambda xs, dt: (np.concatenate(xs) if len(xs) else np.zeros(0, dt))
    return Archive(
        name=name, table=table, words=np.concatenate(words_l),
        word_off=np.array(word_off, np.uint64), nodes=np.concatenate(nodes_l),
        node_off=np.array(node_off, np.uint64),
        ptr_word=np.concatenate(ptr_w), ptr_region=np.concatenate(ptr_r),
        ptr_offset=np.concatenate(ptr_o), decoy_word=np.concatenate(dec_w),
        fp_mask=L.FP_ALL & ~L.FP_GRID_X, graph_tmpl=graph_tmpl,
        tmpl_graph=np.array(tmpl_graph, np.uint32),
        ovr=cat(ovr_l, L.OVR32), ovr_off=np.array(ovr_off, np.uint64),
        govr=cat(govr_l, L.GRID_OVR), govr_off=np.array(govr_off, np.uint64),
        new_base=new_base, map_rank=map_rank, n_ranks=n_ranks,
        patch=cat(patch_l, L.PATCH), patch_off=np.array(patch_off, np.uint64),
        batch_sizes=list(batch_sizes))


# ------------------------------------------------------------------------------------
# flat archives (configs 1, 4): one graph
# ------------------------------------------------------------------------------------
def make_flat_archive(name, seed, n_alloc, size_hi, p_ptr, p_decoy, rest, n_nodes=0,
                      n_words=0, map_kind="shift", size_lo=4096, table_kind="granule"):
    rng = np.random.default_rng(seed)
    table = make_table(rng, n_alloc, size_lo, size_hi, kind=table_kind)
    if n_nodes:
        lens = rng.integers(1, 33, n_nodes).astype(np.int64) * 8  # 8..256 B
        nd = np.zeros(n_nodes, L.NODE)
        nd["kernel_id"] = rng.integers(1, 1 << 63, n_nodes, dtype=np.uint64)
        nd["grid"] = rng.integers(1, 128, (n_nodes, 3)).astype(np.uint32)
        nd["block"][:, 0] = rng.choice([64, 128, 256, 512], n_nodes)
        nd["block"][:, 1:] = 1
        nd["blob_len"] = lens
        nd["flags"] = 0
        n_words = int(lens.sum() // 8)
    else:
        nd = np.zeros(0, L.NODE)
    words, pidx, preg, poff, didx = fill_words(rng, n_words, table, p_ptr, p_decoy, rest)
    if map_kind == "shift":  # one common shift, a multiple of 2 MiB, out of the old span
        new_base = (table["base"] - U64(0x4F0000000000))[None, :].copy()
    elif map_kind == "region_shift":  # distinct shift per region, disjoint from the old span
        i = np.arange(n_alloc, dtype=np.uint64)
        new_base = (U64(0x200000000000) + (table["base"] - U64(OLD_BASE0))
                    + (i + U64(1)) * U64(ALIGN))[None, :].copy()
    else:
        raise ValueError(map_kind)
    z64 = np.zeros(2, np.uint64)
    return Archive(
        name=name, table=table, words=words,
        word_off=np.array([0, n_words], np.uint64), nodes=nd,
        node_off=np.array([0, len(nd)], np.uint64),
        ptr_word=pidx, ptr_region=preg, ptr_offset=poff, decoy_word=didx,
        fp_mask=L.FP_ALL, graph_tmpl=np.zeros(1, np.uint32), tmpl_graph=np.zeros(1, np.uint32),
        ovr=np.zeros(0, L.OVR32), ovr_off=z64.copy(), govr=np.zeros(0, L.GRID_OVR),
        govr_off=z64.copy(), new_base=new_base, map_rank=None, n_ranks=0,
        patch=np.zeros(0, L.PATCH), patch_off=np.zeros(1, np.uint64))


# ------------------------------------------------------------------------------------
# the five configurations
# ------------------------------------------------------------------------------------
CONFIG_NAMES = {1: "tiny", 2: "dense_decode", 3: "moe_decode", 4: "scan_stress", 5: "fleet"}


def make_config(idx, **kw):
    """Config 1..5 at full size; keyword overrides shrink it (same structure, same seed).
    Recognised overrides: n_alloc, n_words (4), n_nodes (1), layers, batch_sizes, n_maps,
    bucket_edges (2: batch sizes up to which each topology bucket reaches), table_kind (4)."""
    seed = SEED0 + idx
    if idx == 1:
        return make_flat_archive("tiny", seed, kw.get("n_alloc", 256), 64 * MiB, 0.25, 0.05, "mix",
                                 n_nodes=kw.get("n_nodes", 512), map_kind="shift")
    if idx == 2:
        return make_model_archive("dense_decode", seed, kw.get("layers", 36), 16,
                                  kw.get("n_alloc", 4096), kw.get("size_hi", 1024 * MiB),
                                  kw.get("batch_sizes", default_batch_sizes()),
                                  kw.get("n_maps", 1), "permute",
                                  bucket_edges=kw.get("bucket_edges", (8, 128)))
    if idx == 3:
        return make_model_archive("moe_decode", seed, kw.get("layers", 94), 28,
                                  kw.get("n_alloc", 16384), 64 * MiB,
                                  kw.get("batch_sizes", default_batch_sizes()),
                                  kw.get("n_maps", 8), "rank_shift", comm_slots=(9, 21),
                                  n_ranks=kw.get("n_ranks", 8))
    if idx == 4:
        return make_flat_archive("scan_stress", seed, kw.get("n_alloc", 1 << 20), 64 * MiB, 0.10,
                                 0.05, "rand64", n_words=kw.get("n_words", 1 << 27),
                                 map_kind="region_shift", table_kind=kw.get("table_kind", "granule"))
    if idx == 5:
        # same template set as config 2 (same seed => same table, graphs, overrides)
        return make_model_archive("fleet", SEED0 + 2, kw.get("layers", 36), 16,
                                  kw.get("n_alloc", 4096), kw.get("size_hi", 1024 * MiB),
                                  kw.get("batch_sizes", default_batch_sizes()),
                                  kw.get("n_maps", 256), "permute")
    raise ValueError(f"no config {idx}")
