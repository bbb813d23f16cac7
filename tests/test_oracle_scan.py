"""Pins for the oracle's pointer scan (CPU only).

The scan has a plain definition (interval membership in a sorted table), so the oracle is
pinned by: a pure-Python brute force written here, the oracle's own linear-search form,
numpy's searchsorted, the generator's planted ground truth (every planted pointer found,
no base-1 / base+size decoy flagged) and hand-made boundary cases.
"""
import numpy as np
import pytest

from synth import layout as L
from tests.cases import small


def py_scan(words, table):
    """Independent statement: test every interval for every word."""
    out = []
    for j, w in enumerate(int(x) for x in words):
        for i, (b, s) in enumerate((int(t["base"]), int(t["size"])) for t in table):
            if b <= w < b + s:
                out.append((j, i, w - b))
    return out


def as_tuples(relocs):
    return [(int(r["word"]), int(r["region"]), int(r["offset"])) for r in relocs]


def mk_table(pairs):
    t = np.zeros(len(pairs), L.ALLOC)
    for i, (b, s) in enumerate(pairs):
        t[i] = (b, s)
    return t


def test_random_tiny_against_python_brute_force(oracle):
    rng = np.random.default_rng(7)
    for trial in range(200):
        A = int(rng.integers(1, 9))
        sizes = rng.integers(1, 40, A)
        gaps = rng.integers(0, 6, A)  # gap 0 => touching intervals
        bases = 1000 + np.concatenate([[0], np.cumsum(sizes[:-1] + gaps[:-1])])
        table = mk_table(list(zip(bases.tolist(), sizes.tolist())))
        assert oracle.table_validate(table)[0] == 0
        W = int(rng.integers(0, 65))
        words = rng.integers(990, int(bases[-1] + sizes[-1]) + 10, W).astype(np.uint64)
        got, cnt = oracle.scan(words, table)
        ref = py_scan(words, table)
        assert cnt == len(ref)
        assert as_tuples(got) == ref
        brute, bcnt = oracle.scan_brute(words, table)
        assert bcnt == cnt and as_tuples(brute) == ref


def test_boundary_cases(oracle):
    table = mk_table([(0x1000, 0x100), (0x1100, 0x10), (0x2000, 1), (2**64 - 0x100, 0xFF)])
    assert oracle.table_validate(table)[0] == 0
    words = np.array(
        [0x0FFF, 0x1000, 0x10FF, 0x1100, 0x110F, 0x1110, 0x1FFF, 0x2000, 0x2001, 0,
         2**64 - 0x101, 2**64 - 0x100, 2**64 - 2, 2**64 - 1], np.uint64)
    got, cnt = oracle.scan(words, table)
    assert as_tuples(got) == [
        (1, 0, 0), (2, 0, 0xFF), (3, 1, 0), (4, 1, 0xF), (7, 2, 0), (11, 3, 0), (12, 3, 0xFE)]
    assert cnt == 7
    # word equal to a touching boundary belongs to the upper interval (index 3 above)
    # one allocation, no words, no allocations
    one = mk_table([(500, 8)])
    assert as_tuples(oracle.scan(np.array([499, 500, 507, 508], np.uint64), one)[0]) == [
        (1, 0, 0), (2, 0, 7)]
    assert oracle.scan(np.zeros(0, np.uint64), one)[1] == 0
    assert oracle.scan(np.array([1, 2, 3], np.uint64), mk_table([]))[1] == 0


def test_capacity_is_respected(oracle):
    table = mk_table([(100, 50)])
    words = np.arange(90, 160, dtype=np.uint64)
    got, cnt = oracle.scan(words, table, capacity=7)
    assert cnt == 50 and len(got) == 7
    assert as_tuples(got) == [(10 + k, 0, k) for k in range(7)]


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_ground_truth_planted_pointers_and_decoys(oracle, idx):
    ar = small(idx)
    assert oracle.table_validate(ar.table)[0] == 0
    got, cnt = oracle.scan(ar.words, ar.table)
    # every planted pointer found with its region and offset, nothing else flagged
    assert cnt == len(ar.ptr_word) == len(got)
    assert np.array_equal(got["word"].astype(np.int64), ar.ptr_word)
    assert np.array_equal(got["region"], ar.ptr_region)
    assert np.array_equal(got["offset"], ar.ptr_offset)
    # decoys really are base-1 / base+size values and none is flagged
    dec = ar.words[ar.decoy_word]
    ends = ar.table["base"] + ar.table["size"]
    assert np.all(np.isin(dec + np.uint64(1), ar.table["base"]) | np.isin(dec, ends))
    assert len(ar.decoy_word) > 0
    assert not np.isin(ar.decoy_word, got["word"].astype(np.int64)).any()


@pytest.mark.parametrize("idx", [1, 4])
def test_equals_linear_search_and_searchsorted(oracle, idx):
    ar = small(idx)
    words = ar.words[:20000]
    got, cnt = oracle.scan(words, ar.table)
    if idx == 1:
        brute, bcnt = oracle.scan_brute(words, ar.table)
        assert bcnt == cnt and np.array_equal(brute, got)
    # library form: upper_bound - 1, then one range check
    i = np.searchsorted(ar.table["base"], words, side="right").astype(np.int64) - 1
    ok = i >= 0
    ii = np.where(ok, i, 0)
    ok &= (words - ar.table["base"][ii]) < ar.table["size"][ii]
    assert np.array_equal(np.flatnonzero(ok), got["word"].astype(np.int64))
    assert np.array_equal(ii[ok].astype(np.uint32), got["region"])


def test_table_validate(oracle):
    good = mk_table([(10, 5), (15, 5), (30, 1)])
    assert oracle.table_validate(good) == (0, 0xFFFFFFFF)
    assert oracle.table_validate(mk_table([(10, 5), (14, 5)])) == (-2, 1)  # overlap
    assert oracle.table_validate(mk_table([(10, 5), (10, 5)])) == (-2, 1)  # not strictly ascending
    assert oracle.table_validate(mk_table([(10, 0)])) == (-2, 0)  # empty range
    assert oracle.table_validate(mk_table([(2**64 - 4, 4)])) == (-2, 0)  # end wraps to 0
    assert oracle.table_validate(mk_table([(2**64 - 4, 3)]))[0] == 0
    assert oracle.table_validate(mk_table([(30, 1), (10, 5)])) == (-2, 1)


def test_reloc_segment(oracle):
    ar = small(2)
    got, _ = oracle.scan(ar.words, ar.table)
    off = oracle.reloc_segment(got, ar.word_off)
    assert off[0] == 0 and off[-1] == len(got)
    ref = np.searchsorted(got["word"].astype(np.uint64), ar.word_off, side="left")
    assert np.array_equal(off, ref.astype(np.uint64))
    # graphs sharing a template blob have equally many relocs
    per_graph = np.diff(off.astype(np.int64))
    for t in range(ar.n_templates):
        assert len(set(per_graph[ar.graph_tmpl == t])) == 1


# ---- scan at 4-byte stride (variant for pointers at 4-byte alignment) -----------------------
def test_stride4_worked_example(oracle):
    # units 0x00000000 0x00000001 0x00000005 0x00000003 0x00000000: the four positions read
    # 0x1_00000000, 0x5_00000001, 0x3_00000005, 0x0_00000003
    table = mk_table([(0x1_0000_0000, 0x10), (0x3_0000_0000, 0x20)])
    relocs, count = oracle.scan_stride4(np.array([0, 1, 5, 3, 0], np.uint32), table)
    assert count == 2 and as_tuples(relocs) == [(0, 0, 0), (2, 1, 5)]
    for n in (0, 1):  # fewer than two units: no position at all
        assert oracle.scan_stride4(np.zeros(n, np.uint32), table)[1] == 0
    assert oracle.scan_stride4(np.array([0, 1], np.uint32), table)[1] == 1  # exactly one position


def test_stride4_python_brute_force(oracle):
    rng = np.random.default_rng(11)
    for trial in range(100):
        A = int(rng.integers(1, 6))
        bases = np.sort(rng.choice(1 << 12, A, replace=False).astype(np.uint64)) << np.uint64(24)
        table = mk_table([(int(b), int(rng.integers(1, 1 << 24))) for b in bases])
        units = rng.integers(0, 1 << 32, int(rng.integers(2, 60)), dtype=np.uint32)
        # plant values at odd and even positions
        for _ in range(int(rng.integers(0, 8))):
            q = int(rng.integers(0, len(units) - 1))
            i = int(rng.integers(0, A))
            v = int(table["base"][i]) + int(rng.integers(0, int(table["size"][i])))
            units[q], units[q + 1] = v & 0xFFFFFFFF, v >> 32
        vals = [int(units[q]) | (int(units[q + 1]) << 32) for q in range(len(units) - 1)]
        relocs, count = oracle.scan_stride4(units, table)
        assert as_tuples(relocs) == py_scan(vals, table) and count == len(relocs)


@pytest.mark.parametrize("idx", [1, 2, 4])
def test_stride4_even_and_odd_positions_are_two_aligned_scans(oracle, idx):
    """Even positions are the 8-byte words of the array, odd positions the 8-byte words of the
    array with its first unit dropped: the 4-byte-stride result is the merge of two scans."""
    ar = small(idx)
    units = np.ascontiguousarray(ar.words).view(np.uint32)[: 2 * min(len(ar.words), 50000)].copy()
    # move every fifth planted pointer of the range half a word up, so that odd positions hit too
    for j in ar.ptr_word[::5]:
        if 2 * j + 2 < len(units):
            units[2 * j + 1], units[2 * j + 2], units[2 * j] = units[2 * j], units[2 * j + 1], 0
    relocs, count = oracle.scan_stride4(units, ar.table)
    even, _ = oracle.scan(units.view(np.uint64), ar.table)
    odd, _ = oracle.scan(units[1:-1].copy().view(np.uint64), ar.table)
    assert count == len(even) + len(odd) and len(odd) > 0
    got_even = relocs[relocs["word"] % 2 == 0]
    got_odd = relocs[relocs["word"] % 2 == 1]
    assert np.array_equal(got_even["word"], 2 * even["word"]) and np.array_equal(got_odd["word"], 2 * odd["word"] + 1)
    for f in ("region", "offset"):
        assert np.array_equal(got_even[f], even[f]) and np.array_equal(got_odd[f], odd[f])
    assert np.all(np.diff(relocs["word"].astype(np.int64)) > 0)
