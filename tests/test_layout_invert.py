"""Inverse of a base map (the relaxation of Section 4.1.1 read backwards: pointers into the new
layout are taken back to the captured one).  Pins of the oracle's definition, then the
library's host call against it.  No GPU needed."""
import numpy as np
import pytest

import paper_2604_06664_amd as fdy
from synth import layout as L
from tests.cases import small


def mk_table(pairs):
    t = np.zeros(len(pairs), L.ALLOC)
    for i, (b, s) in enumerate(pairs):
        t[i] = (b, s)
    return t


def test_worked_example(oracle):
    table = mk_table([(0x1000, 0x100), (0x2000, 0x80), (0x5000, 0x10)])
    new_base = np.array([0x9000, 0x3000, 0x3080], np.uint64)  # regions 1 and 2 touch
    inv_t, inv_b, inv_r = oracle.layout_invert(table, new_base)
    assert inv_t["base"].tolist() == [0x3000, 0x3080, 0x9000]
    assert inv_t["size"].tolist() == [0x80, 0x10, 0x100]
    assert inv_b.tolist() == [0x2000, 0x5000, 0x1000]
    assert inv_r.tolist() == [1, 2, 0]


def test_inverse_of_inverse_is_the_original(oracle):
    for idx in (1, 2, 3, 4, 5):
        ar = small(idx)
        for m in range(min(ar.n_maps, 3)):
            inv_t, inv_b, inv_r = oracle.layout_invert(ar.table, ar.new_base[m])
            assert oracle.table_validate(inv_t)[0] == 0
            back_t, back_b, back_r = oracle.layout_invert(inv_t, inv_b)
            assert np.array_equal(back_t, ar.table)
            assert np.array_equal(back_b, ar.new_base[m])
            assert np.array_equal(inv_r[back_r], np.arange(ar.n_alloc))


def test_scan_of_the_new_layout_finds_the_planted_pointers(oracle):
    """Ground truth from the generator: word ptr_word[k] holds base[ptr_region] + ptr_offset.
    Placed in the new layout by hand, the scan against the inverted table must name the entry
    that stands for that region, with the same offset."""
    ar = small(2)
    new_base = ar.new_base[0]
    inv_t, inv_b, inv_r = oracle.layout_invert(ar.table, new_base)
    with np.errstate(over="ignore"):
        moved = new_base[ar.ptr_region] + ar.ptr_offset
    relocs, count = oracle.scan(moved, inv_t)
    assert count == len(moved)
    assert np.array_equal(inv_r[relocs["region"]], ar.ptr_region)
    assert np.array_equal(relocs["offset"], ar.ptr_offset)
    with np.errstate(over="ignore"):
        assert np.array_equal(inv_b[relocs["region"]] + relocs["offset"], ar.words[ar.ptr_word])


def test_layouts_without_a_way_back(oracle):
    table = mk_table([(0x1000, 0x100), (0x2000, 0x80)])
    assert oracle.layout_invert(table, np.array([0x5000, 0x5080], np.uint64)) is None  # overlap
    assert oracle.layout_invert(table, np.array([0x5000, 0x5000], np.uint64)) is None  # same place
    assert oracle.layout_invert(table, np.array([0x5000, 0x5100], np.uint64)) is not None  # touching
    assert oracle.layout_invert(table, np.array([2**64 - 0x100, 0x10], np.uint64)) is None  # wraps
    assert oracle.layout_invert(table, np.array([2**64 - 0x101, 0x10], np.uint64)) is not None


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_library_matches_oracle(oracle, idx):
    ar = small(idx)
    for m in range(min(ar.n_maps, 3)):
        want = oracle.layout_invert(ar.table, ar.new_base[m])
        rc, inv_t, inv_b, inv_r = fdy.fdy_layout_invert(ar.table, ar.new_base[m])
        assert rc == 0
        assert np.array_equal(inv_t, want[0]) and np.array_equal(inv_b, want[1]) and np.array_equal(inv_r, want[2])


def test_library_error_paths(oracle):
    table = mk_table([(0x1000, 0x100), (0x2000, 0x80)])
    for nb in ([0x5000, 0x5080], [0x5000, 0x5000], [2**64 - 0x100, 0x10], [0x5000, 0x5100], [2**64 - 0x101, 0x10]):
        nb = np.array(nb, np.uint64)
        rc = fdy.fdy_layout_invert(table, nb, check=False)[0]
        assert rc == (fdy.FDY_ERR_TABLE if oracle.layout_invert(table, nb) is None else 0)
    bad = mk_table([(0x2000, 0x80), (0x1000, 0x100)])
    assert fdy.fdy_layout_invert(bad, np.array([0, 0x1000], np.uint64), check=False)[0] == fdy.FDY_ERR_TABLE
    assert fdy.fdy_layout_invert(mk_table([]), np.zeros(0, np.uint64))[0] == 0
    L_ = fdy.lib()
    assert L_.fdy_layout_invert(None, None, 3, None, None, None) == fdy.FDY_ERR_INVALID_ARG
