"""Capture-window replay of a recorded layout in a new address range (Section 4.1.1, Section 5.1:
allocations keep their distance from the start of the range, whatever the start is).  Pins of
the oracle's definition, then the library's host call against it.  No GPU needed."""
import numpy as np
import pytest

import paper_2604_06664_amd as fdy
from synth import layout as L
from tests.cases import small

CODES = {"table": fdy.FDY_ERR_TABLE, "order": fdy.FDY_ERR_ORDER, "capacity": fdy.FDY_ERR_CAPACITY}


def mk_table(pairs):
    t = np.zeros(len(pairs), L.ALLOC)
    for i, (b, s) in enumerate(pairs):
        t[i] = (b, s)
    return t


def test_worked_example(oracle):
    # recorded in a range that started at 0x1000: distances 0x0, 0x200, 0x1000
    rec = mk_table([(0x1000, 0x100), (0x1200, 0x80), (0x2000, 0x10)])
    nb = oracle.layout_replay(rec, 0x1000, 0x7000_0000, 0x1010)
    assert nb.tolist() == [0x7000_0000, 0x7000_0200, 0x7000_1000]
    # the last allocation ends 0x1010 bytes behind the start: one byte less does not hold it
    assert isinstance(oracle.layout_replay(rec, 0x1000, 0x7000_0000, 0x100F), str)
    assert oracle.layout_replay(rec, 0x1000, 0x7000_0000, 0x100F) == "capacity"
    # a range whose first 0x100 bytes are taken cannot take an allocation at distance 0
    assert oracle.layout_replay(rec, 0x1000, 0x7000_0000, 0x2000, new_used=1) == "order"
    # recorded from a start of 0xF00 the first distance is 0x100: 0x100 taken bytes are fine
    assert oracle.layout_replay(rec, 0xF00, 0, 0x2000, new_used=0x100).tolist() == [0x100, 0x300, 0x1100]
    assert oracle.layout_replay(rec, 0xF00, 0, 0x2000, new_used=0x101) == "order"
    assert oracle.layout_replay(rec, 0x1001, 0, 0x2000) == "table"  # starts below its own range
    assert oracle.layout_replay(mk_table([(0x2000, 0x10), (0x1000, 0x10)]), 0, 0, 1 << 40) == "table"
    assert len(oracle.layout_replay(mk_table([]), 5, 6, 0)) == 0


def test_end_of_the_address_space(oracle):
    rec = mk_table([(0x1000, 0x100)])
    top = (1 << 64) - 0x100
    # placed at the very top the allocation would end at 2^64, which no valid table holds
    assert oracle.layout_replay(rec, 0x1000, top, 0x100) == "capacity"
    assert oracle.layout_replay(rec, 0x1000, top - 1, 0x100).tolist() == [top - 1]


@pytest.mark.parametrize("idx", [1, 2, 3, 5])
def test_distances_sizes_and_validity_are_kept(oracle, idx):
    """The replayed layout is the recorded one moved as a whole: equal distances, a valid table,
    and rebasing with it is a pure shift (so scan, materialize with this base map, scan against the
    placed table gives the same regions and offsets)."""
    ar = small(idx)
    start = int(ar.table["base"][0]) - 0x4000
    span = int(ar.table["base"][-1] + ar.table["size"][-1]) - start
    new_start = 0x2000_0000_0000
    nb = oracle.layout_replay(ar.table, start, new_start, span)
    with np.errstate(over="ignore"):
        assert np.array_equal(nb - np.uint64(new_start), ar.table["base"] - np.uint64(start))
    placed = ar.table.copy()
    placed["base"] = nb
    assert oracle.table_validate(placed)[0] == 0
    relocs, _ = oracle.scan(ar.words, ar.table)
    with np.errstate(over="ignore"):
        moved = nb[relocs["region"]] + relocs["offset"]
        assert np.array_equal(moved - ar.words[relocs["word"]],
                              np.full(len(relocs), (new_start - start) % (1 << 64), np.uint64))
    again, cnt = oracle.scan(moved, placed)
    assert cnt == len(relocs)
    assert np.array_equal(again["region"], relocs["region"]) and np.array_equal(again["offset"], relocs["offset"])
    assert oracle.layout_replay(ar.table, start, new_start, span - 1) == "capacity"


def test_library_matches_oracle(oracle):
    rng = np.random.default_rng(77)
    seen = set()
    for trial in range(400):
        n = int(rng.integers(0, 6))
        size = rng.integers(1, 1 << 12, n).astype(np.uint64)
        gap = rng.integers(0, 1 << 10, n).astype(np.uint64)
        first = int(rng.integers(0, 1 << 16))
        base = first + np.concatenate([[0], np.cumsum(size + gap)[:-1]]).astype(np.uint64) if n else np.zeros(0, np.uint64)
        rec = mk_table(list(zip(base.tolist(), size.tolist())))
        if n and trial % 9 == 0:
            rec = rec[::-1].copy()  # not ascending
        recorded_start = first - int(rng.integers(-8, 64)) if n else 0
        recorded_start = max(recorded_start, 0)
        new_start = int(rng.choice([0, 1 << 30, (1 << 64) - (1 << 14), (1 << 64) - 1 - int(size.sum() + gap.sum()) if n else 0]))
        new_capacity = int(rng.choice([0, 1 << 10, 1 << 14, 1 << 40]))
        new_used = int(rng.choice([0, 0, 1, 64, 1 << 20]))
        want = oracle.layout_replay(rec, recorded_start, new_start, new_capacity, new_used)
        rc, nb = fdy.fdy_layout_replay(rec, recorded_start, new_start, new_capacity, new_used, check=False)
        if isinstance(want, str):
            assert rc == CODES[want], (trial, want, rc)
            assert not nb.any()  # not written on error
            seen.add(want)
        else:
            assert rc == 0 and np.array_equal(nb, want), trial
            seen.add("ok")
    assert seen == {"ok", "table", "order", "capacity"}
    assert fdy.lib().fdy_layout_replay(None, 3, 0, 0, 0, 0, None) == fdy.FDY_ERR_INVALID_ARG
