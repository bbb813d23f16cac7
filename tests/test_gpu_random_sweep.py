"""Seeded random sweep of the scan, the fused scan + rebase and the scan at 4-byte stride against
the oracle (GPU).

Table shapes the fixed configurations do not have (clusters of tiny allocations, a few huge
ones, touching ranges, spans from a few KiB to most of the address space, granule-aligned layouts
whose lines mostly take the compact forms, with pointers spread evenly or aimed at the lines that
do not), candidate
densities from none to all, word counts on both sides of sub-tile, group and chunk
boundaries and of the small/large kernel variants, and several sizes of the LDS level."""
import numpy as np
import pytest

from synth import layout as L

pytestmark = pytest.mark.gpu


def random_table(rng, A, shape):
    if shape == "uniform":
        size = rng.integers(1, 1 << 20, A).astype(np.uint64)
        gap = rng.integers(0, 1 << 12, A).astype(np.uint64)
    elif shape == "clustered":  # runs of tiny touching allocations between large ones
        size = np.where(rng.random(A) < 0.9, rng.integers(1, 64, A), rng.integers(1 << 24, 1 << 34, A)).astype(np.uint64)
        gap = np.where(rng.random(A) < 0.7, 0, rng.integers(0, 1 << 30, A)).astype(np.uint64)
    elif shape == "huge":  # sizes and gaps beyond 32 bits: no table line can be packed
        size = rng.integers(1 << 33, 1 << 40, A).astype(np.uint64)
        gap = rng.integers(0, 1 << 36, A).astype(np.uint64)
    elif shape == "aligned":  # allocator-like: aligned blocks, a few of them far beyond 4 GiB, so
        # that the packed table copy needs its per-line shift (and some lines several shifts)
        k = rng.choice([9, 12, 21], A).astype(np.uint64)
        size = rng.integers(1, 1 << 12, A).astype(np.uint64) << k
        big = rng.random(A) < 0.05
        size = np.where(big, rng.integers(1 << 12, 1 << 17, A).astype(np.uint64) << np.uint64(21), size)
        gap = (rng.integers(0, 4, A).astype(np.uint64) << k)
    elif shape.startswith("granular"):  # a layout of whole mapping granules: 2 MiB-aligned bases, sizes in
        # 512-byte steps up to 64 MiB, which the 32-byte forms of the table lines and of the first key level
        # hold; a few odd sizes (such a line only fits the 64-byte form) and a few regions of 8 GiB and more
        # (the table itself) leave marked lines and nodes among the packed ones
        size = rng.integers(8, 1 << 17, A).astype(np.uint64) << np.uint64(9)
        size = np.where(rng.random(A) < 0.02, size + rng.integers(1, 512, A).astype(np.uint64), size)
        size = np.where(rng.random(A) < 0.003, rng.integers(1 << 33, 1 << 36, A).astype(np.uint64), size)
        gran = np.uint64(1 << 21)
        gap = (size + gran - np.uint64(1)) // gran * gran - size + (rng.integers(0, 3, A).astype(np.uint64) << np.uint64(21))
    else:  # "wide": a span of most of the 64-bit space (key shift at its largest)
        size = rng.integers(1, 1 << 30, A).astype(np.uint64)
        gap = (rng.integers(0, 1 << 62, A) // max(A, 1)).astype(np.uint64)
    start = np.concatenate([[0], np.cumsum(size + gap)[:-1]]).astype(np.uint64)
    t = np.zeros(A, L.ALLOC)
    first = np.uint64(rng.integers(1, 1 << 40))
    if shape == "aligned" or shape.startswith("granular"):
        first = first >> np.uint64(21) << np.uint64(21)
    t["base"], t["size"] = first + start, size
    return t


def random_words(rng, W, table, density, skew=False):
    words = rng.integers(0, 1 << 64, W, dtype=np.uint64)
    A = len(table)
    idx = np.flatnonzero(rng.random(W) < density)
    reg = rng.integers(0, A, len(idx))
    if skew:  # most pointers into the few odd or huge regions (their lines are the marked ones)
        special = np.flatnonzero((table["size"] % np.uint64(512) != 0) | (table["size"] >= np.uint64(1 << 33)))
        if len(special):
            reg = np.where(rng.random(len(idx)) < 0.8, special[rng.integers(0, len(special), len(idx))], reg)
    kind = rng.integers(0, 6, len(idx))
    off = (rng.random(len(idx)) * table["size"][reg]).astype(np.uint64)
    off = np.minimum(off, table["size"][reg] - np.uint64(1))
    off = np.where(kind == 0, np.uint64(0), off)
    off = np.where(kind == 1, table["size"][reg] - np.uint64(1), off)
    off = np.where(kind == 2, table["size"][reg], off)  # one past the end
    words[idx] = table["base"][reg] + off
    words[idx[kind == 3]] = table["base"][reg[kind == 3]] - np.uint64(1)  # one below
    return words


CASES = [  # (words, allocations, shape, density, top_log2)
    (700, 1, "uniform", 0.5, 14), (5000, 3, "huge", 0.9, 14), (4096, 17, "clustered", 1.0, 2),
    (8191, 300, "wide", 0.3, 14), (8193, 300, "clustered", 0.05, 5), (16384, 5000, "uniform", 0.0, 14),
    (40001, 5000, "clustered", 0.6, 8), (100000, 70000, "uniform", 0.2, 10), (100000, 70000, "huge", 0.4, 12),
    (262144, 200000, "clustered", 0.33, 14), (262145, 200000, "wide", 0.15, 13), (300000, 16385, "uniform", 0.25, 11),
    (1 << 20, 131073, "clustered", 0.1, 14), (1 << 20, 9, "huge", 1.0, 14),
    (4096 * 512 - 1, 1000, "uniform", 0.02, 14), (4096 * 512 + 513, 300000, "clustered", 0.2, 14),
    (16384 * 512 + 513, 70000, "uniform", 0.1, 14),
    (300000, 70000, "aligned", 0.3, 14), (1 << 20, 200000, "aligned", 0.15, 12), (50000, 40, "aligned", 0.5, 3),
    (1 << 20, 200000, "granular", 0.15, 14), (600000, 150000, "granular_skew", 0.3, 14),
    (300000, 70000, "granular", 0.3, 10), (200000, 131080, "granular_skew", 0.9, 14),
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_random_scan_and_rebase(oracle, case):
    import torch

    assert torch.cuda.is_available()
    import paper_2604_06664_amd as fdy
    from tests.support import session
    from tests.test_gpu_parity import oracle_rebase

    W, A, shape, density, top_log2 = CASES[case]
    rng = np.random.default_rng(1000 + case)
    table = random_table(rng, A, shape)
    assert oracle.table_validate(table)[0] == 0
    words = random_words(rng, W, table, density, skew=shape.endswith("skew"))
    new_base = rng.integers(0, 1 << 64, A, dtype=np.uint64)
    print(f"[sweep] case {case}: W={W} A={A} {shape} density={density} top_log2={top_log2}", flush=True)
    old = fdy.tune_get(fdy.TUNE_SCAN_TOP_LOG2)
    try:
        fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, top_log2)
        ref, rcnt = oracle.scan(words, table)
        got, cnt, status = session.scan(words, table)
        assert status == 0 and cnt == rcnt and np.array_equal(got, ref)
        out_ref, _ = oracle_rebase(oracle, words, table, new_base)
        out, ocnt, ostatus = session.scan_rebase(words, table, new_base)
        assert ostatus == 0 and ocnt == rcnt and np.array_equal(out, out_ref)
        # the same bytes at 4-byte stride, with every third planted value moved half a word up
        units = words.view(np.uint32).copy()
        for j in np.flatnonzero((words >= table["base"][0]) & (words <= table["base"][-1]))[::3]:
            if 2 * j + 2 < len(units):
                units[2 * j + 1], units[2 * j + 2], units[2 * j] = units[2 * j], units[2 * j + 1], 0
        if W % 2:
            units = units[:-1]  # an even and an odd number of units both occur over the cases
        ref4, rcnt4 = oracle.scan_stride4(units, table)
        got4, cnt4, status4 = session.scan_stride4(units, table)
        assert status4 == 0 and cnt4 == rcnt4 and np.array_equal(got4, ref4)
    finally:
        fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, old)
