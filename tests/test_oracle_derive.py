"""Pins for the oracle's override derivation, the SAVE side of templating (CPU only).

Pins: a pure-Python brute force written here; a numpy count of differing 32-bit halves; the
round trip "template + derived overrides = the captured graph" done with numpy stores; on
the model-shaped archives the derived lists against the generator's own override lists
(every derived entry is one of the generator's, and a generator entry that is missing
carries the template's value) and, through the oracle's materialize under the old bases,
against the captured words; a template has no overrides; size mismatch and capacity.
"""
import numpy as np
import pytest

from synth import MatProblem
from synth import layout as L
from tests.cases import small


def brute(words, word_off, graph_tmpl, tmpl_graph):
    """Byte for byte, in Python integers."""
    raw = np.ascontiguousarray(words, np.uint64).view(np.uint8)
    out, off = [], [0]
    for g in range(len(graph_tmpl)):
        s = int(tmpl_graph[int(graph_tmpl[g])])
        a0, b0 = int(word_off[g]) * 8, int(word_off[s]) * 8
        n = (int(word_off[g + 1]) - int(word_off[g])) * 8
        assert n == (int(word_off[s + 1]) - int(word_off[s])) * 8
        for o in range(0, n, 4):
            va = int.from_bytes(bytes(raw[a0 + o:a0 + o + 4]), "little")
            vb = int.from_bytes(bytes(raw[b0 + o:b0 + o + 4]), "little")
            if va != vb:
                out.append((o, va))
        off.append(len(out))
    return out, off


def random_case(rng, G, T, max_words):
    """G graphs in T groups; graphs of a group share a length and differ in a few halves."""
    lens = rng.integers(0, max_words + 1, T)
    graph_tmpl = np.concatenate([np.arange(T), rng.integers(0, T, G - T)]).astype(np.uint32)
    rng.shuffle(graph_tmpl)
    # dense ids in order of first appearance, as the fingerprint would number them
    order, remap = [], {}
    for t in graph_tmpl:
        if int(t) not in remap:
            remap[int(t)] = len(order)
            order.append(int(t))
    graph_tmpl = np.array([remap[int(t)] for t in graph_tmpl], np.uint32)
    lens = lens[order]
    tmpl_graph = np.array([int(np.flatnonzero(graph_tmpl == t)[0]) for t in range(T)], np.uint32)
    word_off = np.concatenate([[0], np.cumsum(lens[graph_tmpl])]).astype(np.uint64)
    words = np.zeros(int(word_off[-1]), np.uint64)
    for g in range(G):
        s = int(tmpl_graph[graph_tmpl[g]])
        n = int(lens[graph_tmpl[g]])
        a = int(word_off[g])
        if g == s:
            words[a:a + n] = rng.integers(0, 1 << 64, n, dtype=np.uint64)
        else:
            words[a:a + n] = words[int(word_off[s]):int(word_off[s]) + n]
            h = words[a:a + n].view(np.uint32)
            k = int(rng.integers(0, min(2 * n, 9) + 1)) if n else 0
            for pos in rng.choice(2 * n, k, replace=False) if k else []:
                h[pos] = rng.integers(0, 1 << 32, dtype=np.uint64)  # may equal the old value
    return words, word_off, graph_tmpl, tmpl_graph


def test_brute_force_on_random_small_cases(oracle):
    rng = np.random.default_rng(11)
    for _ in range(40):
        G = int(rng.integers(1, 12))
        T = int(rng.integers(1, G + 1))
        words, word_off, gt, tg = random_case(rng, G, T, 40)
        ovr, off = oracle.derive_overrides(words, word_off, gt, tg)
        want, woff = brute(words, word_off, gt, tg)
        assert [int(x) for x in off] == woff
        assert [(int(o["byte_off"]), int(o["value"])) for o in ovr] == want


@pytest.mark.parametrize("idx", [2, 3, 5])
def test_counts_round_trip_and_generator_lists(oracle, idx):
    ar = small(idx)
    ovr, off = oracle.derive_overrides(ar.words, ar.word_off, ar.graph_tmpl, ar.tmpl_graph)
    assert int(off[-1]) == len(ovr) and int(off[0]) == 0
    halves = ar.words.view(np.uint32)
    for g in range(ar.n_graphs):
        s = int(ar.tmpl_graph[ar.graph_tmpl[g]])
        a, b = int(ar.word_off[g]) * 2, int(ar.word_off[g + 1]) * 2
        ts = int(ar.word_off[s]) * 2
        mine = ovr[int(off[g]):int(off[g + 1])]
        # count: numpy's own comparison of the 32-bit halves
        assert len(mine) == int((halves[a:b] != halves[ts:ts + (b - a)]).sum())
        assert np.all(np.diff(mine["byte_off"].astype(np.int64)) > 0) and np.all(mine["byte_off"] % 4 == 0)
        # round trip: template + derived overrides = the captured graph
        rebuilt = halves[ts:ts + (b - a)].copy()
        rebuilt[mine["byte_off"] // 4] = mine["value"]
        assert np.array_equal(rebuilt, halves[a:b])
        # against the generator's privileged lists
        gen = ar.ovr[int(ar.ovr_off[g]):int(ar.ovr_off[g + 1])]
        gen_map = {int(o["byte_off"]): int(o["value"]) for o in gen}
        for o in mine:
            assert gen_map.get(int(o["byte_off"])) == int(o["value"])
        derived = set(int(x) for x in mine["byte_off"])
        for bo, v in gen_map.items():
            if bo not in derived:
                assert int(halves[ts + bo // 4]) == v  # same as the template: nothing to store
        if g == s:
            assert len(mine) == 0
    # through materialize under the old bases: the captured words come back
    relocs, _ = oracle.scan(ar.words, ar.table)
    mp = MatProblem.from_archive(ar, relocs, oracle.reloc_segment(relocs, ar.word_off))
    kw = {n: getattr(mp, n) for n in MatProblem.ARRAYS}
    kw.update(ovr=ovr, ovr_off=off, new_base=ar.table["base"][None, :].copy(), map_rank=None)
    out, _ = oracle.materialize(MatProblem(n_ranks=0, **kw), want_dims=False)
    assert np.array_equal(out[0], ar.words)


def test_errors_and_capacity(oracle):
    words = np.arange(10, dtype=np.uint64)
    with pytest.raises(ValueError):  # graph 1 (4 words) against a template of 6 words
        oracle.derive_overrides(words, [0, 6, 10], [0, 0], [0])
    with pytest.raises(ValueError):  # template id out of range
        oracle.derive_overrides(words, [0, 5, 10], [0, 1], [0])
    full, off = oracle.derive_overrides(words, [0, 5, 10], [0, 0], [0])
    assert int(off[2]) == 5 and len(full) == 5  # low halves differ, high halves are all zero
    cut, off2 = oracle.derive_overrides(words, [0, 5, 10], [0, 0], [0], capacity=3)
    assert np.array_equal(off, off2) and np.array_equal(cut, full[:3])
    none, off3 = oracle.derive_overrides(np.zeros(0, np.uint64), [0], np.zeros(0, np.uint32), np.zeros(0, np.uint32))
    assert len(none) == 0 and list(off3) == [0]
