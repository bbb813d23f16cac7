"""Pins for the oracle's template materialization (CPU only).

Pins: identity (scan then materialize under the old bases, with each graph's overrides,
reproduces every captured graph blob), round trip (rebase, scan against the new table,
rebase back), pure shift, equal maps, a word-at-a-time brute force (the oracle's own and a
pure-Python one written here), patches touch only patched words, stage precedence.
"""
import numpy as np
import pytest

from synth import MatProblem
from synth import layout as L
from tests.cases import small


def problem(oracle, ar, **kw):
    relocs, cnt = oracle.scan(ar.words, ar.table)
    assert cnt == len(relocs)
    roff = oracle.reloc_segment(relocs, ar.word_off)
    return MatProblem.from_archive(ar, relocs, roff, **kw)


def with_maps(mp, new_base, map_rank="keep"):
    kw = {n: getattr(mp, n) for n in MatProblem.ARRAYS}
    kw["new_base"] = new_base
    if map_rank != "keep":
        kw["map_rank"] = map_rank
    return MatProblem(n_ranks=mp.n_ranks if kw["map_rank"] is not None else 0, **kw)


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_identity_reproduces_every_captured_graph(oracle, idx):
    ar = small(idx)
    mp = with_maps(problem(oracle, ar), ar.table["base"][None, :].copy(), map_rank=None)
    out, dims = oracle.materialize(mp)
    assert out.shape == (1, len(ar.words))
    assert np.array_equal(out[0], ar.words)  # byte for byte, all graphs
    if len(ar.nodes):
        assert np.array_equal(dims[:, :3], ar.nodes["grid"])
        assert np.array_equal(dims[:, 3:], ar.nodes["block"])


@pytest.mark.parametrize("idx", [1, 2, 4, 5])
def test_round_trip_through_a_new_map(oracle, idx):
    ar = small(idx)
    mp = problem(oracle, ar)
    out, _ = oracle.materialize(mp, want_dims=False)
    for m in range(min(ar.n_maps, 3)):
        # new table = same regions at their new bases, sorted by new base
        order = np.argsort(ar.new_base[m], kind="stable")
        nt = np.zeros(ar.n_alloc, L.ALLOC)
        nt["base"] = ar.new_base[m][order]
        nt["size"] = ar.table["size"][order]
        assert oracle.table_validate(nt)[0] == 0
        rel2, cnt2 = oracle.scan(out[m], nt)
        assert cnt2 == len(ar.ptr_word)  # the same words are pointers in the new layout
        # materialize the rebased archive back to the old bases: every graph its own template
        back_base = np.empty(ar.n_alloc, np.uint64)
        back_base[:] = ar.table["base"][order]  # region k of the new table is old region order[k]
        G = ar.n_graphs
        mp2 = MatProblem(
            src_words=out[m], src_word_off=ar.word_off, src_nodes=ar.nodes, src_node_off=ar.node_off,
            relocs=rel2, src_reloc_off=oracle.reloc_segment(rel2, ar.word_off),
            tmpl_graph=np.arange(G), graph_tmpl=np.arange(G), ovr=np.zeros(0, L.OVR32),
            ovr_off=np.zeros(G + 1), govr=np.zeros(0, L.GRID_OVR), govr_off=np.zeros(G + 1),
            new_base=back_base[None, :], map_rank=None, n_ranks=0, patch=np.zeros(0, L.PATCH),
            patch_off=np.zeros(1))
        back, _ = oracle.materialize(mp2, want_dims=False)
        assert np.array_equal(back[0], ar.words)


def test_pure_shift_moves_exactly_the_pointer_words(oracle):
    ar = small(1)
    mp = problem(oracle, ar)
    out, _ = oracle.materialize(mp, want_dims=False)
    shift = ar.new_base[0][0] - ar.table["base"][0]
    assert np.all(ar.new_base[0] - ar.table["base"] == shift) and shift % np.uint64(2 << 20) == 0
    diff = out[0] - ar.words
    is_ptr = np.zeros(len(ar.words), bool)
    is_ptr[ar.ptr_word] = True
    assert np.all(diff[is_ptr] == shift) and np.all(diff[~is_ptr] == 0)


def test_equal_maps_give_equal_outputs(oracle):
    ar = small(5)
    mp = problem(oracle, ar)
    nb = np.repeat(ar.new_base[1:2], 3, axis=0)
    out, _ = oracle.materialize(with_maps(mp, nb), want_dims=False)
    assert np.array_equal(out[0], out[1]) and np.array_equal(out[0], out[2])
    ref, _ = oracle.materialize(mp, want_dims=False)
    assert np.array_equal(out[0], ref[1])
    assert not np.array_equal(ref[0], ref[1])


def py_materialize(mp):
    """Independent pure-Python word-at-a-time form."""
    out = np.zeros((mp.M, mp.out_words_per_map()), np.uint64)
    M64 = (1 << 64) - 1
    for m in range(mp.M):
        pos = 0
        for g in range(mp.G):
            t = int(mp.graph_tmpl[g])
            s = int(mp.tmpl_graph[t])
            w0, w1 = int(mp.src_word_off[s]), int(mp.src_word_off[s + 1])
            rel = {int(r["word"]): r for r in mp.relocs[int(mp.src_reloc_off[s]):int(mp.src_reloc_off[s + 1])]}
            ov = {int(o["byte_off"]): int(o["value"]) for o in mp.ovr[int(mp.ovr_off[g]):int(mp.ovr_off[g + 1])]}
            pt = {}
            if mp.map_rank is not None:
                row = t * mp.n_ranks + int(mp.map_rank[m])
                pt = {int(p["word"]): int(p["value"]) for p in mp.patch[int(mp.patch_off[row]):int(mp.patch_off[row + 1])]}
            for k in range(w1 - w0):
                v = int(mp.src_words[w0 + k])
                if w0 + k in rel:
                    r = rel[w0 + k]
                    v = (int(mp.new_base[m][int(r["region"])]) + int(r["offset"])) & M64
                if 8 * k in ov:
                    v = (v & ~0xFFFFFFFF & M64) | ov[8 * k]
                if 8 * k + 4 in ov:
                    v = (v & 0xFFFFFFFF) | (ov[8 * k + 4] << 32)
                if k in pt:
                    v = pt[k]
                out[m, pos + k] = v
            pos += w1 - w0
    return out


@pytest.mark.parametrize("idx", [1, 2, 3])
def test_staged_equals_word_at_a_time(oracle, idx):
    kw = {2: dict(layers=2, batch_sizes=[1, 2, 16, 24, 512]),
          3: dict(layers=2, batch_sizes=[4, 16, 24], n_maps=8, n_alloc=512)}.get(idx, {})
    from synth import make_config

    ar = make_config(idx, **kw)
    mp = problem(oracle, ar)
    out, _ = oracle.materialize(mp, want_dims=False)
    assert np.array_equal(out, oracle.materialize_brute(mp))
    assert np.array_equal(out, py_materialize(mp))


def test_rank_patches_touch_only_patched_words(oracle):
    ar = small(3)
    mp = problem(oracle, ar)
    out, _ = oracle.materialize(mp, want_dims=False)
    plain, _ = oracle.materialize(with_maps(mp, mp.new_base, map_rank=None), want_dims=False)
    out_off = np.concatenate([[0], np.cumsum(np.diff(ar.word_off.astype(np.int64))[ar.tmpl_graph[ar.graph_tmpl]])])
    for m in range(ar.n_maps):
        r = int(ar.map_rank[m])
        differs = np.flatnonzero(out[m] != plain[m])
        expect_idx, expect_val = [], []
        for g in range(ar.n_graphs):
            row = int(ar.graph_tmpl[g]) * ar.n_ranks + r
            p = ar.patch[int(ar.patch_off[row]):int(ar.patch_off[row + 1])]
            expect_idx.append(out_off[g] + p["word"].astype(np.int64))
            expect_val.append(p["value"])
        expect_idx, expect_val = np.concatenate(expect_idx), np.concatenate(expect_val)
        assert np.array_equal(out[m][expect_idx], expect_val)
        assert np.isin(differs, expect_idx).all() and len(differs) > 0
    # the stub words of the single-rank capture are not pointers (never in the reloc table)
    stub_words = np.concatenate([
        int(ar.word_off[ar.tmpl_graph[t]]) + ar.patch[int(ar.patch_off[t * ar.n_ranks]):int(ar.patch_off[t * ar.n_ranks + 1])]["word"].astype(np.int64)
        for t in range(ar.n_templates)])
    assert not np.isin(stub_words, mp.relocs["word"].astype(np.int64)).any()


def test_stage_precedence_copy_rebase_override_patch(oracle):
    # one template of 4 words; word 1: reloc + override(low) ; word 2: reloc + override(high) + patch
    words = np.array([11, 0x1000 + 5, 0x1000 + 9, 44], np.uint64)
    table = np.zeros(1, L.ALLOC)
    table[0] = (0x1000, 0x100)
    relocs, _ = oracle.scan(words, table)
    assert relocs["word"].tolist() == [1, 2]
    ovr = np.zeros(3, L.OVR32)
    ovr[0], ovr[1], ovr[2] = (8, 0xAAAA), (20, 0xBBBB), (28, 0xCCCC)
    patch = np.zeros(1, L.PATCH)
    patch[0] = (2, 0, 0xDEADBEEF00000001)
    mp = MatProblem(
        src_words=words, src_word_off=[0, 4], src_nodes=np.zeros(0, L.NODE), src_node_off=[0, 0],
        relocs=relocs, src_reloc_off=[0, 2], tmpl_graph=[0], graph_tmpl=[0, 0], ovr=ovr,
        ovr_off=[0, 0, 3], govr=np.zeros(0, L.GRID_OVR), govr_off=[0, 0, 0],
        new_base=np.array([[0x500000], [0x900000]], np.uint64), map_rank=[1, 0], n_ranks=2,
        patch=patch, patch_off=[0, 0, 1])  # only rank 1 has a patch
    out, _ = oracle.materialize(mp, want_dims=False)
    # map 0 (rank 1, patched), graph 0 (no overrides), graph 1 (overrides)
    assert out[0].tolist() == [11, 0x500005, 0xDEADBEEF00000001, 44,
                               11, 0x500000 & ~0xFFFFFFFF | 0xAAAA, 0xDEADBEEF00000001, 44 | (0xCCCC << 32)]
    # map 1 (rank 0, no patch): word 2 keeps rebase + high-half override
    assert out[1].tolist() == [11, 0x900005, 0x900009, 44,
                               11, 0xAAAA, 0x900009 | (0xBBBB << 32), 44 | (0xCCCC << 32)]
    assert np.array_equal(out, py_materialize(mp))
    assert np.array_equal(out, oracle.materialize_brute(mp))


def test_rebase_wraps_modulo_2_64(oracle):
    words = np.array([0x1000 + 0x20], np.uint64)
    table = np.zeros(1, L.ALLOC)
    table[0] = (0x1000, 0x100)
    relocs, _ = oracle.scan(words, table)
    mp = MatProblem(
        src_words=words, src_word_off=[0, 1], src_nodes=np.zeros(0, L.NODE), src_node_off=[0, 0],
        relocs=relocs, src_reloc_off=[0, 1], tmpl_graph=[0], graph_tmpl=[0], ovr=np.zeros(0, L.OVR32),
        ovr_off=[0, 0], govr=np.zeros(0, L.GRID_OVR), govr_off=[0, 0],
        new_base=np.array([[2**64 - 0x10]], np.uint64), map_rank=None, n_ranks=0,
        patch=np.zeros(0, L.PATCH), patch_off=[0])
    out, _ = oracle.materialize(mp, want_dims=False)
    assert int(out[0, 0]) == 0x10


def test_grid_overrides_in_dims(oracle):
    ar = small(2)
    mp = problem(oracle, ar)
    _, dims = oracle.materialize(mp)
    # template + grid overrides reproduces every captured graph's launch dims
    assert np.array_equal(dims[:, :3], ar.nodes["grid"])
    assert np.array_equal(dims[:, 3:], ar.nodes["block"])
    # and without overrides every graph shows its template's dims
    kw = {n: getattr(mp, n) for n in MatProblem.ARRAYS}
    kw["govr"], kw["govr_off"] = np.zeros(0, L.GRID_OVR), np.zeros(mp.G + 1)
    _, d0 = oracle.materialize(MatProblem(n_ranks=0, **kw))
    N = len(ar.nodes) // ar.n_graphs
    for g in range(ar.n_graphs):
        s = int(ar.tmpl_graph[ar.graph_tmpl[g]])
        assert np.array_equal(d0[g * N:(g + 1) * N, :3], ar.nodes["grid"][s * N:(s + 1) * N])
    assert not np.array_equal(d0, dims)


def test_invalid_inputs_are_rejected(oracle):
    ar = small(1)
    mp = problem(oracle, ar)
    assert oracle.materialize_validate(mp) == 0
    bad = mp.relocs.copy()
    bad["region"][3] = ar.n_alloc
    kw = {n: getattr(mp, n) for n in MatProblem.ARRAYS}
    kw["relocs"] = bad
    assert oracle.materialize_validate(MatProblem(n_ranks=0, **kw)) == -1
    kw["relocs"] = mp.relocs
    kw["graph_tmpl"] = np.array([1], np.uint32)
    with pytest.raises((ValueError, IndexError)):
        oracle.materialize(MatProblem(n_ranks=0, **kw))
