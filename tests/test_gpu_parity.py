"""Parity of the HIP path (through the C-ABI) against the CPU oracle: bit-exact, element by
element.  Everything here needs a real MI355X (`-m gpu`)."""
import numpy as np
import pytest

from synth import MatProblem, make_config
from synth import layout as L
from tests.cases import small

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hip():
    import torch

    assert torch.cuda.is_available(), "gpu tests need a GPU"
    import paper_2604_06664_amd as fdy
    from tests.support import session

    fdy.lib()
    return session


def mk_table(pairs):
    t = np.zeros(len(pairs), L.ALLOC)
    for i, (b, s) in enumerate(pairs):
        t[i] = (b, s)
    return t


def say(msg):
    print(msg, flush=True)


MODES = ((False, True), (True, True), (False, False), (True, False))  # (prepared table, staging area)


# ------------------------------------------------------------------------------------ scan
def check_scan(hip, oracle, words, table, capacity=None, tag=""):
    say(f"[scan] {tag} W={len(words)} A={len(table)} cap={capacity}")
    ref, rcnt = oracle.scan(words, table, capacity)
    cap = len(words) if capacity is None else capacity
    # hierarchy built by the call / by fdy_scan_table_prepare; dense groups staged / searched twice
    for prepared, staging in MODES:
        got, cnt, status = hip.scan(words, table, capacity, prepared=prepared, staging=staging)
        assert cnt == rcnt
        assert np.array_equal(got, ref)
        assert status == (L.ST_CAPACITY if rcnt > cap else 0)
    return got


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_scan_small_configs(hip, oracle, idx):
    ar = small(idx)
    got = check_scan(hip, oracle, ar.words, ar.table, tag=ar.name)
    assert np.array_equal(got["word"].astype(np.int64), ar.ptr_word)  # generator ground truth


def test_scan_edge_cases(hip, oracle):
    ar = small(1)
    one = mk_table([(500, 8)])
    check_scan(hip, oracle, np.zeros(0, np.uint64), ar.table, tag="no words")
    check_scan(hip, oracle, ar.words[:100], mk_table([]), tag="no allocations")
    check_scan(hip, oracle, np.array([499, 500, 507, 508], np.uint64), one, tag="one allocation")
    check_scan(hip, oracle, ar.words[:1], ar.table, tag="one word")
    for n in (2047, 2048, 2049, 4095, 4097, 6001):  # around tile boundaries, odd tails
        check_scan(hip, oracle, ar.words[:n], ar.table, tag="ragged")
    # every word a hit (queue and output completely full), touching intervals, extremes
    dense = mk_table([(0x1000 + 64 * i, 64) for i in range(300)] + [(2**64 - 0x100, 0xFF)])
    rng = np.random.default_rng(3)
    w = (0x1000 + rng.integers(0, 64 * 300, 5000)).astype(np.uint64)
    w[::97] = np.uint64(2**64 - 1)
    w[1::97] = np.uint64(2**64 - 2)
    w[2::97] = np.uint64(0xFFF)
    check_scan(hip, oracle, w, dense, tag="all hits")
    # capacity smaller than the number of hits: count is the need, prefix is written
    check_scan(hip, oracle, w, dense, capacity=1234, tag="overflow")
    check_scan(hip, oracle, w, dense, capacity=0, tag="zero capacity")


def test_scan_hierarchical_levels(hip, oracle):
    """Force the sampled LDS level + in-table refinement on small tables by shrinking the
    LDS budget, so every depth of the hierarchy is exercised at sizes the oracle likes."""
    import paper_2604_06664_amd as fdy

    ar = small(4)  # 65,536 allocations
    old = fdy.tune_get(fdy.TUNE_SCAN_TOP_LOG2)
    try:
        for top_log2 in (1, 3, 8, 11, 12, 13, 14):
            assert fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, top_log2) >= 0
            check_scan(hip, oracle, ar.words[:300000], ar.table, tag=f"top_log2={top_log2}")
            check_scan(hip, oracle, ar.words[:5000], ar.table[:1000], tag=f"A=1000 top_log2={top_log2}")
            check_scan(hip, oracle, ar.words[:5000], ar.table[:1025], tag=f"A=1025 top_log2={top_log2}")
    finally:
        fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, old)


def test_scan_truncated_key_ambiguity(hip, oracle):
    """The LDS level holds truncated keys; candidates whose key equals a sampled base's key
    must be settled on exact bases.  Unaligned bases in a very wide span, words placed just
    below / at / above bases inside the same truncation granule, and a cluster of tiny
    allocations that all share one key."""
    import paper_2604_06664_amd as fdy

    rng = np.random.default_rng(21)
    A = 40000
    base = (np.uint64(0x1000_0000_0005) + np.arange(A, dtype=np.uint64) * np.uint64(1 << 33)
            + rng.integers(0, 4096, A).astype(np.uint64) * np.uint64(8))
    size = np.full(A, 100, np.uint64)
    # a cluster of 3000 16-byte allocations, 16 bytes apart, inside one key granule
    cb = base[100] + np.uint64(1 << 20) + np.arange(3000, dtype=np.uint64) * np.uint64(16)
    allb = np.concatenate([base, cb])
    alls = np.concatenate([size, np.full(3000, 16, np.uint64)])
    order = np.argsort(allb)
    table = np.zeros(len(allb), L.ALLOC)
    table["base"], table["size"] = allb[order], alls[order]
    assert oracle.table_validate(table)[0] == 0
    pick = rng.integers(0, len(table), 60000)
    delta = rng.choice(np.array([-9, -1, 0, 1, 15, 16, 99, 100, 101, 5000], np.int64), 60000)
    words = (table["base"][pick].astype(np.int64) + delta).astype(np.uint64)
    old = fdy.tune_get(fdy.TUNE_SCAN_TOP_LOG2)
    try:
        for top_log2 in (14, 9, 4):
            fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, top_log2)
            check_scan(hip, oracle, words, table, tag=f"ambiguous keys top_log2={top_log2}")
    finally:
        fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, old)


def test_scan_large_input_dense_groups_and_wide_lines(hip, oracle):
    """The large-input kernel variant (two groups of two sub-tiles per wave) on an input long
    enough to select it, with everything that variant handles specially: stretches where every
    word is a pointer (groups beyond the register-resident limit: windowed two-pass path),
    moderate and zero density elsewhere, a ragged tail, and a 200,000-entry table read through
    its packed copy in which some 8-entry lines cannot be packed (an allocation of 5 GiB, a
    gap of 6 GiB) and the last line is partial."""
    rng = np.random.default_rng(77)
    A = 200_003
    size = rng.integers(16, 1 << 16, A).astype(np.uint64)
    gap = rng.integers(0, 4096, A).astype(np.uint64) * np.uint64(16)
    size[::1000] = np.uint64(5 << 30)       # a size that does not fit 32 bits
    gap[500::1000] = np.uint64(6 << 30)     # a line that spans more than 4 GiB
    start = np.concatenate([[0], np.cumsum(size + gap)[:-1]]).astype(np.uint64)
    table = np.zeros(A, L.ALLOC)
    table["base"], table["size"] = np.uint64(0x7E00_0000_1000) + start, size
    assert oracle.table_validate(table)[0] == 0
    W = 16500 * 512 + 777
    words = rng.integers(0, 1 << 20, W).astype(np.uint64)  # small integers: outside the span

    def plant(lo, hi, density):
        idx = lo + np.flatnonzero(rng.random(hi - lo) < density)
        reg = rng.integers(0, A, len(idx))
        kind = rng.integers(0, 8, len(idx))
        off = (rng.random(len(idx)) * table["size"][reg]).astype(np.uint64)
        off = np.where(kind == 0, np.uint64(0), off)                            # first byte
        off = np.where(kind == 1, table["size"][reg] - np.uint64(1), off)       # last byte
        off = np.where(kind == 2, table["size"][reg], off)                      # one past: no hit
        words[idx] = table["base"][reg] + off
        words[idx[kind == 3]] = table["base"][reg[kind == 3]] - np.uint64(1)    # one below

    plant(0, 2_000_000, 0.30)
    plant(2_000_000, 2_600_000, 1.0)     # dense: every group overflows the register path
    plant(2_600_000, 2_600_700, 0.0)
    plant(3_000_000, 3_001_536, 1.0)     # a dense island of three sub-tiles
    plant(5_000_000, W, 0.12)
    plant(W - 777, W, 1.0)               # dense ragged tail
    got = check_scan(hip, oracle, words, table, tag="large variant")
    assert len(got) > 1_000_000


def test_prepared_table_is_reused_and_checked(hip, oracle):
    """One prepared table serves calls of every scan entry point one after the other (each call
    must leave the counters it used zeroed), for inputs of different sizes, including inputs of
    no words; a table prepared for something else is refused on the device."""
    import paper_2604_06664_amd as fdy
    import torch

    ar = small(4)  # 65,536 allocations, 2^20 words
    nb = ar.new_base[0]
    base = hip.ScanPointersRebaseRun(ar.words, ar.table, nb, prepared=True)
    sizes = [len(ar.words), 70001, 0, 16384, 5000, 1 << 19]
    for rep in range(2):
        for n in sizes:
            say(f"[prepared] rep {rep} n={n}")
            ref, rcnt = oracle.scan(ar.words[:n], ar.table)
            want = oracle_rebase(oracle, ar.words[:n], ar.table, nb)[0] if n else np.zeros(0, np.uint64)
            for kind in ("scan", "out", "rebase"):
                base.n_words = n
                base.d_count.fill_(-1)
                base.d_status.zero_()
                base.d_out.fill_(0xEE)
                base.d_relocs.fill_(0xEE)
                if kind == "scan":
                    fdy.fdy_scan_pointers(base.d_words, n, base.d_table, base.n_alloc, base.d_relocs,
                                          base.capacity, base.d_count, base.d_prepared, base.d_ws,
                                          base.ws_bytes, base.d_status)
                elif kind == "out":
                    base.launch()
                else:
                    fdy.fdy_scan_rebase(base.d_words, n, base.d_table, base.n_alloc, base.d_new_base,
                                        base.d_out, base.d_count, base.d_prepared, base.d_ws, base.ws_bytes,
                                        base.d_status)
                torch.cuda.synchronize()
                assert int(base.d_status.item()) == 0 and int(base.d_count.item()) == rcnt, kind
                if kind != "rebase":
                    assert np.array_equal(fdy.to_host(base.d_relocs, hip.RELOC, rcnt), ref), kind
                if kind != "scan":
                    assert np.array_equal(fdy.to_host(base.d_out, np.uint64, n), want), kind
    # the counters are zero again (header of the state: 64 counters behind the hierarchy)
    # refused: more words than prepared for, another table address, another table size
    other = fdy.to_device(ar.table)
    for words, table, n_alloc in ((len(ar.words) + 1, base.d_table, base.n_alloc),
                                  (1000, other, base.n_alloc), (1000, base.d_table, base.n_alloc - 8)):
        base.d_status.zero_()
        base.d_relocs.fill_(0xEE)
        big = fdy.device_bytes((len(ar.words) + 1) * 8)
        fdy.fdy_scan_pointers(big, words, table, n_alloc, base.d_relocs, base.capacity, base.d_count,
                              base.d_prepared, base.d_ws, base.ws_bytes, base.d_status)
        torch.cuda.synchronize()
        assert int(base.d_status.item()) == L.ST_BAD_PREPARED
        assert bool((base.d_relocs[:4096] == 0xEE).all())
    # and still good afterwards
    got, cnt, status, out = (base.__setattr__("n_words", len(ar.words)), base.d_status.zero_(), base.launch(),
                             base.result())[-1]
    ref, rcnt = oracle.scan(ar.words, ar.table)
    assert status == 0 and cnt == rcnt and np.array_equal(got, ref)


def test_scan_bounded_wait_is_reported_not_hung(hip):
    """Host-forced error path: with a spin limit of 0 a workgroup that finds its predecessor
    unfinished gives up at once, raises FDY_ST_SPIN and still terminates."""
    import paper_2604_06664_amd as fdy

    ar = small(4)
    old = fdy.tune_set(fdy.TUNE_SCAN_SPIN_LIMIT, 0)
    try:
        _, _, status = hip.scan(ar.words, ar.table)
        assert status & ~(L.ST_SPIN | L.ST_CAPACITY) == 0  # terminated; only these bits possible
    finally:
        fdy.tune_set(fdy.TUNE_SCAN_SPIN_LIMIT, old)
    got, cnt, status = hip.scan(ar.words, ar.table)
    assert status == 0 and cnt == len(ar.ptr_word)


def test_scan_argument_errors(hip):
    import paper_2604_06664_amd as fdy
    import torch

    ar = small(1)
    run = hip.ScanRun(ar.words, ar.table)
    bad = fdy.fdy_scan_pointers(run.d_words.data_ptr() + 8, run.n_words - 1, run.d_table, run.n_alloc,
                                run.d_relocs, run.capacity, run.d_count, None, run.d_ws, run.ws_bytes,
                                run.d_status, check=False)
    assert bad == fdy.FDY_ERR_INVALID_ARG
    assert fdy.fdy_scan_pointers(run.d_words, run.n_words, run.d_table, run.n_alloc, run.d_relocs,
                                 run.capacity, run.d_count, None, run.d_ws,
                                 fdy.fdy_scan_workspace_bytes(run.n_words, run.n_alloc) - 1, run.d_status,
                                 check=False) == fdy.FDY_ERR_WORKSPACE
    assert fdy.fdy_scan_pointers(run.d_words, 1 << 32, run.d_table, run.n_alloc, run.d_relocs,
                                 run.capacity, run.d_count, None, run.d_ws, run.ws_bytes, run.d_status,
                                 check=False) == fdy.FDY_ERR_INVALID_ARG
    torch.cuda.synchronize()


# --------------------------------------------------------------------- override derivation
def check_derive(hip, oracle, words, word_off, gt, tg, capacity=None, tag=""):
    say(f"[derive] {tag} W={len(words)} G={len(gt)} T={len(tg)} cap={capacity}")
    ref, roff = oracle.derive_overrides(words, word_off, gt, tg, capacity)
    got, off, status = hip.derive_overrides(words, word_off, gt, tg, capacity)
    assert np.array_equal(off, roff)
    assert np.array_equal(got, ref)
    cap = 2 * len(words) if capacity is None else capacity
    assert status == (L.ST_CAPACITY if int(roff[-1]) > cap else 0)
    return got, off


def test_derive_overrides_random_and_edge_cases(hip, oracle):
    from tests.test_oracle_derive import random_case

    rng = np.random.default_rng(19)
    for k in range(12):
        G = int(rng.integers(1, 40))
        T = int(rng.integers(1, G + 1))
        words, word_off, gt, tg = random_case(rng, G, T, 5000 if k % 3 == 0 else 300)  # several tiles
        check_derive(hip, oracle, words, word_off, gt, tg, tag=f"random {k}")
    words, word_off, gt, tg = random_case(rng, 30, 4, 4100)
    _, off = check_derive(hip, oracle, words, word_off, gt, tg, tag="for capacity")
    total = int(off[-1])
    if total > 2:
        check_derive(hip, oracle, words, word_off, gt, tg, capacity=total // 2, tag="overflow")
    check_derive(hip, oracle, words, word_off, gt, tg, capacity=0, tag="zero capacity")
    # every half differs (output twice the number of words), exact tile multiples, empty graphs
    a = np.arange(4096, dtype=np.uint64) * np.uint64(0x100000001)
    both = np.concatenate([a, ~a, a[:0], a])
    check_derive(hip, oracle, both, [0, 4096, 8192, 8192, 8192, 12288], [0, 0, 1, 1, 0], [0, 2], tag="all differ")
    check_derive(hip, oracle, np.zeros(0, np.uint64), [0], np.zeros(0, np.uint32), np.zeros(0, np.uint32),
                 tag="no graphs")
    # bad inputs are flagged, not faulting: template id out of range, sizes that differ
    got, off, status = hip.derive_overrides(a, [0, 2048, 4096], [0, 7], [0])
    assert status == L.ST_BAD_INDEX and len(got) == 0 and list(off) == [0, 0, 0]
    got, off, status = hip.derive_overrides(a, [0, 2048, 4096, 4096], [0, 0, 0], [0])
    assert status == L.ST_BAD_SIZE and int(off[-1]) == 4096  # graph 2 (empty) skipped, graph 1 compared


@pytest.mark.parametrize("idx", [2, 3, 5])
def test_derive_overrides_archives_and_round_trip(hip, oracle, idx):
    """Fingerprint -> derive -> materialize under the old bases, all on the GPU, gives back the
    captured words of every graph: the generator's privileged override lists are not needed."""
    ar = small(idx)
    mask = L.FP_ALL & ~L.FP_GRID_X
    _, tid, tg, _ = hip.fingerprint(ar.nodes, ar.node_off, mask)
    assert np.array_equal(tid, ar.graph_tmpl) and np.array_equal(tg, ar.tmpl_graph)
    ovr, off = check_derive(hip, oracle, ar.words, ar.word_off, tid, tg, tag=ar.name)
    mp = problem(oracle, ar)
    kw = {n: getattr(mp, n) for n in MatProblem.ARRAYS}
    kw.update(ovr=ovr, ovr_off=off, new_base=ar.table["base"][None, :].copy(), map_rank=None)
    mp2 = MatProblem(n_ranks=0, **kw)
    out, _, status = hip.materialize(mp2, want_dims=False)
    assert status == 0 and np.array_equal(out[0], ar.words)


# ------------------------------------------------------------------- scan at 4-byte stride
def check_scan4(hip, oracle, units, table, capacity=None, tag=""):
    units = np.ascontiguousarray(units, np.uint32)
    say(f"[scan stride 4] {tag} units={len(units)} A={len(table)} cap={capacity}")
    ref, rcnt = oracle.scan_stride4(units, table, capacity)
    cap = max(len(units) - 1, 0) if capacity is None else capacity
    for prepared, staging in MODES:
        got, cnt, status = hip.scan_stride4(units, table, capacity, prepared=prepared, staging=staging)
        assert cnt == rcnt
        assert np.array_equal(got, ref)
        assert status == (L.ST_CAPACITY if rcnt > cap else 0)
    return got


def units_with_odd_pointers(ar, n_words=None):
    """The archive's words as 32-bit units, every fifth planted pointer moved half a word up."""
    n = len(ar.words) if n_words is None else min(n_words, len(ar.words))
    units = np.ascontiguousarray(ar.words[:n]).view(np.uint32).copy()
    for j in ar.ptr_word[::5]:
        if 2 * j + 2 < len(units):
            units[2 * j + 1], units[2 * j + 2], units[2 * j] = units[2 * j], units[2 * j + 1], 0
    return units


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_scan_stride4_small_configs(hip, oracle, idx):
    ar = small(idx)
    units = units_with_odd_pointers(ar)
    got = check_scan4(hip, oracle, units, ar.table, tag=ar.name)
    assert (got["word"] % 2 == 1).sum() > 0 and (got["word"] % 2 == 0).sum() > 0
    check_scan4(hip, oracle, units[:-1], ar.table, tag=ar.name + " odd unit count")


def test_scan_stride4_edge_cases(hip, oracle):
    import paper_2604_06664_amd as fdy

    ar = small(4)  # 65,536 allocations
    units = units_with_odd_pointers(ar, 300000)
    for n in (0, 1, 2, 3, 511, 512, 513, 514, 1024, 1025, 1026, 2049, 4097, 70001, 131073):
        check_scan4(hip, oracle, units[:n], ar.table, tag="ragged")
    # a pointer on every seam: the last position of a sub-tile takes its high half from the next
    # sub-tile, the last lane of a 16-byte piece row from the next row, the last position of all
    # from the last unit
    t = mk_table([(0x7000_0000_0000, 0x1000), (0x7000_0010_0000, 0x40)])
    rng = np.random.default_rng(3)
    u = rng.integers(0, 1 << 31, 5000, dtype=np.uint32)  # high halves below the table: no stray hit
    for q, v in ((255, 0x7000_0000_0008), (511, 0x7000_0000_0FFF), (767, 0x7000_0010_0000), (1023, 0x7000_0010_003F),
                 (1535, 0x7000_0000_0000), (4998, 0x7000_0010_0001)):
        u[q], u[q + 1] = v & 0xFFFFFFFF, v >> 32
    got = check_scan4(hip, oracle, u, t, tag="seams")
    assert got["word"].tolist() == [255, 511, 767, 1023, 1535, 4998]
    check_scan4(hip, oracle, u, t, capacity=3, tag="capacity 3")
    # no table: nothing is a pointer
    got, cnt, status = hip.scan_stride4(u, t[:0])
    assert cnt == 0 and status == 0
    # (nearly) every position a hit: the windowed path
    wide = mk_table([(0, 1 << 63), (1 << 63, (1 << 63) - 1)])
    check_scan4(hip, oracle, rng.integers(0, 1 << 32, 9001, dtype=np.uint32), wide, tag="all hits")
    old = fdy.tune_get(fdy.TUNE_SCAN_TOP_LOG2)
    try:
        for top_log2 in (3, 9):
            fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, top_log2)
            check_scan4(hip, oracle, units[:200001], ar.table, tag=f"top_log2={top_log2}")
    finally:
        fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, old)
    # misaligned array refused on the host
    run = hip.ScanStride4Run(u, t)
    rc = fdy.fdy_scan_pointers_stride4(run.d_words.data_ptr() + 4, 100, run.d_table, 2, run.d_relocs, 10,
                                       run.d_count, None, run.d_ws, run.ws_bytes, run.d_status, check=False)
    assert rc == fdy.FDY_ERR_INVALID_ARG


def test_scan_stride4_large_input(hip, oracle):
    """2^23 units against 2^16 allocations: the large-input kernel shape (two groups of two
    sub-tiles per wave), several chunks per workgroup."""
    ar = make_config(4, n_words=(1 << 22) + 4096, n_alloc=1 << 16)
    units = units_with_odd_pointers(ar)
    got = check_scan4(hip, oracle, units, ar.table, tag="large")
    assert len(got) > 300_000


# ------------------------------------------------------------------- fused scan + rebase
def oracle_rebase(oracle, words, table, new_base):
    """What fdy_scan_rebase must produce, from the oracle's own scan and materialize: one
    source graph holding all the words, one base map, no overrides, no patches."""
    words = np.ascontiguousarray(words, np.uint64)
    relocs, cnt = oracle.scan(words, table)
    woff = np.array([0, len(words)], np.uint64)
    mp = MatProblem(
        src_words=words, src_word_off=woff, src_nodes=np.zeros(0, L.NODE), src_node_off=[0, 0],
        relocs=relocs, src_reloc_off=oracle.reloc_segment(relocs, woff), tmpl_graph=[0], graph_tmpl=[0],
        ovr=np.zeros(0, L.OVR32), ovr_off=[0, 0], govr=np.zeros(0, L.GRID_OVR), govr_off=[0, 0],
        new_base=np.ascontiguousarray(new_base, np.uint64).reshape(1, -1), map_rank=None, n_ranks=0,
        patch=np.zeros(0, L.PATCH), patch_off=[0])
    out, _ = oracle.materialize(mp, want_dims=False)
    return out[0], cnt


def check_rebase(hip, oracle, words, table, new_base, tag="", in_place=False):
    say(f"[scan_rebase] {tag} W={len(words)} A={len(table)} in_place={in_place}")
    ref, rcnt = oracle_rebase(oracle, words, table, new_base) if len(words) else (np.zeros(0, np.uint64), 0)
    for prepared in (False, True):
        got, cnt, status = hip.scan_rebase(words, table, new_base, in_place=in_place, prepared=prepared)
        assert cnt == rcnt and status == 0
        assert np.array_equal(got, ref)


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_scan_rebase_small_configs(hip, oracle, idx):
    ar = small(idx)
    check_rebase(hip, oracle, ar.words, ar.table, ar.new_base[0], tag=ar.name)
    check_rebase(hip, oracle, ar.words, ar.table, ar.new_base[0], tag=ar.name + " in place", in_place=True)


def test_scan_rebase_edge_cases(hip, oracle):
    import paper_2604_06664_amd as fdy

    ar = small(4)  # 65,536 allocations
    nb = ar.new_base[0]
    check_rebase(hip, oracle, np.zeros(0, np.uint64), ar.table, nb, tag="no words")
    check_rebase(hip, oracle, ar.words[:1], ar.table, nb, tag="one word")
    for n in (1023, 1024, 1025, 2047, 4097, 70001):  # group and sub-tile boundaries, odd tails
        check_rebase(hip, oracle, ar.words[:n], ar.table, nb, tag="ragged")
    # no table: a plain copy
    got, cnt, status = hip.scan_rebase(ar.words[:5000], ar.table[:0], nb[:0])
    assert cnt == 0 and status == 0 and np.array_equal(got, ar.words[:5000])
    # every word a hit (groups beyond the queue: windowed path), touching intervals, extremes,
    # sums that wrap mod 2^64
    dense = mk_table([(0x1000 + 64 * i, 64) for i in range(300)] + [(2**64 - 0x100, 0xFF)])
    rng = np.random.default_rng(5)
    w = (0x1000 + rng.integers(0, 64 * 300, 9000)).astype(np.uint64)
    w[::97] = np.uint64(2**64 - 1)
    w[1::97] = np.uint64(2**64 - 2)
    w[2::97] = np.uint64(0xFFF)
    dnb = rng.integers(0, 1 << 64, len(dense), dtype=np.uint64)
    check_rebase(hip, oracle, w, dense, dnb, tag="all hits")
    check_rebase(hip, oracle, w, dense, dnb, tag="all hits in place", in_place=True)
    # every depth of the hierarchy, with the packed table copy and unpackable lines
    old = fdy.tune_get(fdy.TUNE_SCAN_TOP_LOG2)
    try:
        for top_log2 in (3, 9, 12):
            fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, top_log2)
            check_rebase(hip, oracle, ar.words[:200000], ar.table, nb, tag=f"top_log2={top_log2}")
    finally:
        fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, old)
    # overlapping, non-identical input and output ranges are refused on the host
    run = hip.ScanRebaseRun(ar.words[:4096], ar.table, nb)
    rc = fdy.fdy_scan_rebase(run.d_words, 2048, run.d_table, run.n_alloc, run.d_new_base,
                             run.d_words.data_ptr() + 1024 * 8, run.d_count, None, run.d_ws, run.ws_bytes,
                             run.d_status, check=False)
    assert rc == fdy.FDY_ERR_INVALID_ARG


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_scan_rebase_there_and_back(hip, oracle, idx):
    """Rebase into a new layout, then back through the inverted layout (fdy_layout_invert): the
    second pass equals the oracle's rebase of the first pass's output, and every planted
    pointer is its captured value again."""
    import paper_2604_06664_amd as fdy

    ar = small(idx)
    nb = ar.new_base[0]
    there, cnt, status = hip.scan_rebase(ar.words, ar.table, nb)
    assert status == 0 and cnt == len(ar.ptr_word)
    rc, inv_t, inv_b, inv_r = fdy.fdy_layout_invert(ar.table, nb)
    want = oracle.layout_invert(ar.table, nb)
    assert np.array_equal(inv_t, want[0]) and np.array_equal(inv_b, want[1])
    say(f"[scan_rebase] {ar.name} back through the inverted layout, A={len(inv_t)}")
    back, cnt_back, status = hip.scan_rebase(there, inv_t, inv_b)
    ref, rcnt = oracle_rebase(oracle, there, inv_t, inv_b)
    assert status == 0 and cnt_back == rcnt and np.array_equal(back, ref)
    assert cnt_back >= cnt  # every moved pointer is found again (plus words that happen to lie there)
    assert np.array_equal(back[ar.ptr_word], ar.words[ar.ptr_word])
    # relocations of the new layout name the captured regions through inv_region
    relocs, n, status = hip.scan(there, inv_t)
    assert status == 0 and n == cnt_back
    at = np.searchsorted(relocs["word"], ar.ptr_word)
    assert np.array_equal(relocs["word"][at], ar.ptr_word.astype(np.uint32))
    assert np.array_equal(inv_r[relocs["region"][at]], ar.ptr_region)
    assert np.array_equal(relocs["offset"][at], ar.ptr_offset)


# ------------------------------------------- scan with rebased output (table and copy in one pass)
def check_scan_out(hip, oracle, words, table, new_base, capacity=None, tag=""):
    """fdy_scan_pointers_rebase = the oracle's scan (table) and the oracle's scan + materialize of
    one own-template graph under one base map (output)."""
    say(f"[scan_pointers_rebase] {tag} W={len(words)} A={len(table)} cap={capacity}")
    ref, rcnt = oracle.scan(words, table, capacity)
    want, _ = oracle_rebase(oracle, words, table, new_base) if len(words) else (np.zeros(0, np.uint64), 0)
    cap = len(words) if capacity is None else capacity
    for prepared, staging in MODES:
        got, cnt, status, out = hip.scan_pointers_rebase(words, table, new_base, capacity, prepared=prepared,
                                                         staging=staging)
        assert cnt == rcnt
        assert np.array_equal(got, ref)
        assert status == (L.ST_CAPACITY if rcnt > cap else 0)
        assert np.array_equal(out, want)


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_scan_pointers_rebase_small_configs(hip, oracle, idx):
    ar = small(idx)
    check_scan_out(hip, oracle, ar.words, ar.table, ar.new_base[0], tag=ar.name)


def test_scan_pointers_rebase_edge_cases(hip, oracle):
    import paper_2604_06664_amd as fdy

    ar = small(4)  # 65,536 allocations
    nb = ar.new_base[0]
    check_scan_out(hip, oracle, np.zeros(0, np.uint64), ar.table, nb, tag="no words")
    check_scan_out(hip, oracle, ar.words[:1], ar.table, nb, tag="one word")
    for n in (511, 512, 513, 1023, 1025, 4097, 16384, 16385, 70001):  # sub-tile, group, chunk edges
        check_scan_out(hip, oracle, ar.words[:n], ar.table, nb, tag="ragged")
    check_scan_out(hip, oracle, ar.words[:5000], ar.table[:0], nb[:0], tag="no table: a plain copy")
    check_scan_out(hip, oracle, ar.words[:300000], ar.table, nb, capacity=1000, tag="capacity exceeded")
    # every word a hit (dense groups: windowed path with staged entries), touching intervals,
    # extremes, sums that wrap mod 2^64
    dense = mk_table([(0x1000 + 64 * i, 64) for i in range(300)] + [(2**64 - 0x100, 0xFF)])
    rng = np.random.default_rng(5)
    w = (0x1000 + rng.integers(0, 64 * 300, 9000)).astype(np.uint64)
    w[::97] = np.uint64(2**64 - 1)
    w[1::97] = np.uint64(2**64 - 2)
    w[2::97] = np.uint64(0xFFF)
    dnb = rng.integers(0, 1 << 64, len(dense), dtype=np.uint64)
    check_scan_out(hip, oracle, w, dense, dnb, tag="all hits")
    # a large input (the large-chunk kernel) whose first part is dense and whose rest is sparse
    big = np.concatenate([w] * 40 + [ar.words[:3_000_000]])
    tb = np.concatenate([dense[:300], ar.table]) if dense["base"][299] < ar.table["base"][0] else ar.table
    nb2 = rng.integers(0, 1 << 64, len(tb), dtype=np.uint64)
    check_scan_out(hip, oracle, big, tb, nb2, tag="large, dense head")
    # overlapping input and output are refused on the host, in place included
    run = hip.ScanPointersRebaseRun(ar.words[:4096], ar.table, nb)
    for out in (run.d_words.data_ptr(), run.d_words.data_ptr() + 1024 * 8):
        rc = fdy.fdy_scan_pointers_rebase(run.d_words, 2048, run.d_table, run.n_alloc, run.d_relocs,
                                          run.capacity, run.d_count, run.d_new_base, out, None, run.d_ws,
                                          run.ws_bytes, run.d_status, check=False)
        assert rc == fdy.FDY_ERR_INVALID_ARG


def test_reloc_segment(hip, oracle):
    ar = small(2)
    run = hip.ScanRun(ar.words, ar.table)
    run.launch()
    relocs, cnt, _ = run.result()
    for bounds in (ar.word_off, np.array([0], np.uint64), np.array([5, 5, 10**9], np.uint64)):
        got, _ = hip.reloc_segment(run.d_relocs, run.d_count, run.capacity, bounds)
        assert np.array_equal(got, oracle.reloc_segment(relocs, bounds))
    # an empty relocation table
    run0 = hip.ScanRun(ar.words[:50], mk_table([(1, 1)]))
    run0.launch()
    got, _ = hip.reloc_segment(run0.d_relocs, run0.d_count, run0.capacity, ar.word_off[:3])
    assert got.tolist() == [0, 0, 0]


# ----------------------------------------------------------------------------- fingerprint
@pytest.mark.parametrize("idx", [1, 2, 3, 5])
def test_fingerprint_small_configs(hip, oracle, idx):
    ar = small(idx)
    for mask in (ar.fp_mask, L.FP_ALL, L.FP_KERNEL_ID | L.FP_BLOB_LEN, L.FP_GRID_Y | L.FP_BLOCK, 0):
        say(f"[fingerprint] {ar.name} mask={mask:#x}")
        keys, tid, tg = oracle.fingerprint(ar.nodes, ar.node_off, mask)
        gk, gt, gg, _ = hip.fingerprint(ar.nodes, ar.node_off, mask)
        assert np.array_equal(gk, keys)
        assert np.array_equal(gt, tid)
        assert np.array_equal(gg, tg)


def test_fingerprint_edge_cases(hip, oracle):
    nodes = small(1).nodes
    # empty graphs, one-node graphs, a graph longer than a workgroup, duplicates out of order
    off = np.array([0, 0, 1, 3, 3, 4, 4 + 300, 4 + 300, 4 + 301], np.uint64)
    nd = np.concatenate([nodes[:4], nodes[:300], nodes[:1]])
    keys, tid, tg = oracle.fingerprint(nd, off, L.FP_ALL)
    gk, gt, gg, _ = hip.fingerprint(nd, off, L.FP_ALL)
    assert np.array_equal(gk, keys) and np.array_equal(gt, tid) and np.array_equal(gg, tg)
    assert tid[0] == tid[3] == tid[6] and tid[1] == tid[7]
    # no graphs at all
    gk, gt, gg, _ = hip.fingerprint(nodes[:0], np.zeros(1, np.uint64), L.FP_ALL)
    assert len(gk) == 0 and len(gg) == 0
    # many graphs (several chunks of the grouping workgroup), few distinct keys
    rng = np.random.default_rng(5)
    pick = rng.integers(0, 7, 2500)
    lens = np.array([3, 1, 4, 1, 5, 9, 2])
    starts = np.concatenate([[0], np.cumsum(lens)])
    nd = np.concatenate([nodes[starts[p]:starts[p] + lens[p]] for p in pick])
    off = np.concatenate([[0], np.cumsum(lens[pick])]).astype(np.uint64)
    keys, tid, tg = oracle.fingerprint(nd, off, L.FP_ALL)
    gk, gt, gg, _ = hip.fingerprint(nd, off, L.FP_ALL, want_tmpl_graph=False)
    assert np.array_equal(gk, keys) and np.array_equal(gt, tid) and gg is None
    _, _, gg, _ = hip.fingerprint(nd, off, L.FP_ALL)
    assert np.array_equal(gg, tg)


def test_fingerprint_many_graphs_and_templates(hip, oracle):
    """The shape of Section 6.4.1: 512 graphs (batch sizes 1..512) in 22 topology groups; then
    sizes around and beyond what the grouping table in LDS holds (8,192 graphs; beyond it the
    table lies in the workspace), with every graph distinct, with few distinct ones, and with
    templates first met late."""
    edges = [1, 2, 4, 8, 16, 24, 32, 48, 64, 96, 128, 160, 192, 224, 256, 288, 320, 352, 384, 416, 448]
    ar = make_config(2, layers=4, batch_sizes=list(range(1, 513)), bucket_edges=edges)
    assert ar.n_graphs == 512 and ar.n_templates == 22
    keys, tid, tg = oracle.fingerprint(ar.nodes, ar.node_off, ar.fp_mask)
    assert np.array_equal(tid, ar.graph_tmpl) and np.array_equal(tg, ar.tmpl_graph)
    gk, gt, gg, _ = hip.fingerprint(ar.nodes, ar.node_off, ar.fp_mask)
    assert np.array_equal(gk, keys) and np.array_equal(gt, tid) and np.array_equal(gg, tg)
    nodes = small(1).nodes
    rng = np.random.default_rng(9)
    for G, distinct in ((8191, 8191), (8192, 8192), (8193, 8193), (8192, 37), (20000, 20000), (70000, 1000),
                        (300000, 3)):
        say(f"[fingerprint] G={G} distinct={distinct}")
        # graph i = one node of the archive with its kernel id replaced by the pick
        pick = rng.integers(0, distinct, G).astype(np.uint64)
        pick[: min(G, distinct)] = rng.permutation(min(G, distinct)).astype(np.uint64)
        nd = np.repeat(nodes[:1], G)
        nd["kernel_id"] = pick + np.uint64(1000)
        off = np.arange(G + 1, dtype=np.uint64)
        keys, tid, tg = oracle.fingerprint(nd, off, L.FP_ALL)
        gk, gt, gg, _ = hip.fingerprint(nd, off, L.FP_ALL)
        assert np.array_equal(gk, keys) and np.array_equal(gt, tid) and np.array_equal(gg, tg)


@pytest.mark.parametrize("idx", [1, 2, 3])
def test_segment_fingerprint_one_launch(hip, oracle, idx):
    """fdy_segment_fingerprint = fdy_reloc_segment + fdy_fingerprint, with the grouping done by
    the last block of the launch (a prepared table supplies its counter) or by a second launch
    (no prepared table); called twice in a row on the same prepared table."""
    import paper_2604_06664_amd as fdy
    import torch

    ar = small(idx)
    relocs, cnt = oracle.scan(ar.words, ar.table)
    roff = oracle.reloc_segment(relocs, ar.word_off)
    keys, tid, tg = oracle.fingerprint(ar.nodes, ar.node_off, ar.fp_mask)
    G = ar.n_graphs
    srun = hip.ScanRun(ar.words, ar.table, prepared=True)
    srun.launch()
    d_word_off, d_nodes, d_node_off = fdy.to_device(ar.word_off), fdy.to_device(ar.nodes), fdy.to_device(ar.node_off)
    for prepared in (srun.d_prepared, None, srun.d_prepared):
        d_roff = fdy.device_bytes((G + 1) * 8, fill=0xEE)
        d_keys, d_tid, d_tg = (fdy.device_bytes(G * 8, fill=0xEE), fdy.device_bytes(G * 4, fill=0xEE),
                               fdy.device_bytes(G * 4, fill=0xEE))
        d_nt = torch.full((1,), -1, dtype=torch.int32, device="cuda:0")
        fdy.fdy_segment_fingerprint(srun.d_relocs, srun.d_count, srun.capacity, d_word_off, d_roff, d_nodes,
                                    d_node_off, G, ar.fp_mask, d_keys, d_tid, d_tg, d_nt, d_prepared=prepared)
        torch.cuda.synchronize()
        nt = int(d_nt.item())
        assert nt == len(tg)
        assert np.array_equal(fdy.to_host(d_roff, np.uint64, G + 1), roff)
        assert np.array_equal(fdy.to_host(d_keys, np.uint64, G), keys)
        assert np.array_equal(fdy.to_host(d_tid, np.uint32, G), tid)
        assert np.array_equal(fdy.to_host(d_tg, np.uint32, nt), tg)
    # the scan still works on the prepared table afterwards
    got, n, st = (srun.launch(), srun.result())[-1]
    assert st == 0 and n == cnt and np.array_equal(got, relocs)


# ----------------------------------------------------------------------------- materialize
def problem(oracle, ar, **kw):
    relocs, _ = oracle.scan(ar.words, ar.table)
    return MatProblem.from_archive(ar, relocs, oracle.reloc_segment(relocs, ar.word_off), **kw)


def check_mat(hip, oracle, mp, tag="", want_dims=True):
    say(f"[materialize] {tag} G={mp.G} M={mp.M} T={mp.T} words/map={mp.out_words_per_map()}")
    ref, rdims = oracle.materialize(mp, want_dims)
    out, dims, status = hip.materialize(mp, want_dims)
    assert status == 0
    assert np.array_equal(out, ref)
    if want_dims:
        assert np.array_equal(dims, rdims)
    return out


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_materialize_small_configs(hip, oracle, idx):
    ar = small(idx)
    mp = problem(oracle, ar)
    check_mat(hip, oracle, mp, tag=ar.name)
    check_mat(hip, oracle, mp, tag=ar.name + " no dims", want_dims=False)


def test_materialize_identity_on_gpu(hip, oracle):
    ar = small(2)
    mp = problem(oracle, ar)
    kw = {n: getattr(mp, n) for n in MatProblem.ARRAYS}
    kw["new_base"] = ar.table["base"][None, :].copy()
    out, dims, status = hip.materialize(MatProblem(n_ranks=0, **kw))
    assert status == 0 and np.array_equal(out[0], ar.words)
    assert np.array_equal(dims[:, :3], ar.nodes["grid"])


def test_materialize_stage_precedence_and_wrap(hip, oracle):
    words = np.array([11, 0x1000 + 5, 0x1000 + 9, 44], np.uint64)
    table = mk_table([(0x1000, 0x100)])
    relocs, _ = oracle.scan(words, table)
    ovr = np.zeros(3, L.OVR32)
    ovr[0], ovr[1], ovr[2] = (8, 0xAAAA), (20, 0xBBBB), (28, 0xCCCC)
    patch = np.zeros(1, L.PATCH)
    patch[0] = (2, 0, 0xDEADBEEF00000001)
    mp = MatProblem(
        src_words=words, src_word_off=[0, 4], src_nodes=np.zeros(0, L.NODE), src_node_off=[0, 0],
        relocs=relocs, src_reloc_off=[0, 2], tmpl_graph=[0], graph_tmpl=[0, 0], ovr=ovr,
        ovr_off=[0, 0, 3], govr=np.zeros(0, L.GRID_OVR), govr_off=[0, 0, 0],
        new_base=np.array([[0x500000], [2**64 - 3]], np.uint64), map_rank=[1, 0], n_ranks=2,
        patch=patch, patch_off=[0, 0, 1])
    out = check_mat(hip, oracle, mp, tag="precedence", want_dims=False)
    assert out[0, 6] == 0xDEADBEEF00000001 and out[1, 1] == 2  # (2^64-3)+5 wraps to 2


def test_materialize_tile_boundaries_and_empty_graphs(hip, oracle):
    """Templates of 0, 1, 2047, 2048, 2049 and 5000 words; overrides and patches placed on
    the first / last word of tiles; outputs referencing templates in scrambled order."""
    rng = np.random.default_rng(11)
    table = small(1).table
    lens = [0, 1, 2047, 2048, 2049, 5000]
    from synth.archive import fill_words

    words, *_ = fill_words(rng, sum(lens), table, 0.3, 0.05, "mix")
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)
    relocs, _ = oracle.scan(words, table)
    roff = oracle.reloc_segment(relocs, off)
    graph_tmpl = np.array([5, 0, 3, 3, 1, 4, 2, 0, 5], np.uint32)
    ovr_l, ovr_off, patch_l, patch_off = [], [0], [], [0]
    for g, t in enumerate(graph_tmpl):
        n = lens[t]
        spots = sorted({b for b in (0, 4, 8 * 2047, 8 * 2047 + 4, 8 * 2048, 8 * 2048 + 4, 8 * n - 4) if 0 <= b < 8 * n})
        o = np.zeros(len(spots), L.OVR32)
        o["byte_off"], o["value"] = spots, rng.integers(0, 2**32, len(spots))
        ovr_l.append(o)
        ovr_off.append(ovr_off[-1] + len(o))
    R = 3
    for t in range(len(lens)):
        for r in range(R):
            n = lens[t]
            spots = sorted({k for k in (0, 2047, 2048, 4095, 4096, n - 1) if 0 <= k < n}) if r != 1 else []
            q = np.zeros(len(spots), L.PATCH)
            q["word"], q["value"] = spots, rng.integers(0, 2**63, len(spots))
            patch_l.append(q)
            patch_off.append(patch_off[-1] + len(q))
    G = len(graph_tmpl)
    mp = MatProblem(
        src_words=words, src_word_off=off, src_nodes=np.zeros(0, L.NODE), src_node_off=np.zeros(len(lens) + 1),
        relocs=relocs, src_reloc_off=roff, tmpl_graph=np.arange(len(lens)), graph_tmpl=graph_tmpl,
        ovr=np.concatenate(ovr_l), ovr_off=ovr_off, govr=np.zeros(0, L.GRID_OVR), govr_off=np.zeros(G + 1),
        new_base=small(1).new_base.repeat(4, axis=0) + np.arange(4, dtype=np.uint64)[:, None] * np.uint64(1 << 30),
        map_rank=[2, 0, 1, 2], n_ranks=R, patch=np.concatenate(patch_l), patch_off=patch_off)
    check_mat(hip, oracle, mp, tag="tile boundaries", want_dims=False)


def replicate_outputs(mp, times):
    """The same problem with every output graph listed `times` times over (lists repeated)."""
    kw = {n: getattr(mp, n) for n in MatProblem.ARRAYS}
    kw["graph_tmpl"] = np.tile(mp.graph_tmpl, times)
    for lst, off in (("ovr", "ovr_off"), ("govr", "govr_off")):
        o = getattr(mp, off).astype(np.int64)
        kw[lst] = np.tile(getattr(mp, lst), times)
        kw[off] = np.concatenate([[0]] + [o[1:] + k * o[-1] for k in range(times)])
    return MatProblem(n_ranks=mp.n_ranks, **kw)


@pytest.mark.parametrize("idx,times", [(2, 128), (2, 129), (3, 300)])
def test_materialize_more_than_1024_graphs(hip, oracle, idx, times):
    """Up to 1024 output graphs the tile launch computes the per-graph prefix sums itself; above
    that a launch of its own does.  8 x 128 = 1024 graphs is the last case of the first kind,
    8 x 129 and 5 x 300 are of the second; with launch dimensions, overrides and rank patches."""
    mp = replicate_outputs(problem(oracle, small(idx), maps=[0, 1] if idx == 3 else None), times)
    check_mat(hip, oracle, mp, tag=f"{mp.G} graphs")


def test_materialize_bad_inputs_are_flagged_not_faulting(hip, oracle):
    import paper_2604_06664_amd as fdy

    ar = small(1)
    mp = problem(oracle, ar)
    # region out of range in one reloc: entry skipped, status bit raised, rest as the oracle
    bad = mp.relocs.copy()
    bad["region"][7] = ar.n_alloc + 5
    kw = {n: getattr(mp, n) for n in MatProblem.ARRAYS}
    kw["relocs"] = bad
    out, _, status = hip.materialize(MatProblem(n_ranks=0, **kw), want_dims=False)
    assert status == L.ST_BAD_INDEX
    ref, _ = oracle.materialize(mp, want_dims=False)
    k = int(bad["word"][7])
    assert out[0, k] == ar.words[k]  # the skipped entry leaves the template word
    ref[0, k] = ar.words[k]
    assert np.array_equal(out, ref)
    # wrong total from the caller: nothing is written
    run = hip.MatRun(mp, want_dims=False)
    run.desc.out_words_per_map = run.wpm - 1
    run.launch()
    out, _, status = run.result()
    assert status & L.ST_BAD_SIZE and np.all(out.view(np.uint8) == 0xCD)
    # template index out of range
    kw["relocs"] = mp.relocs
    run = hip.MatRun(mp, want_dims=False)
    run.dev["graph_tmpl"] = fdy.to_device(np.array([9], np.uint32))
    run.desc = fdy.make_mat_desc(run.dev, n_src_graphs=mp.S, n_templates=mp.T, n_graphs=mp.G, n_maps=mp.M,
                                 n_alloc=mp.A, n_ranks=0, out_words_per_map=run.wpm, out_nodes_total=0)
    run.launch()
    out, _, status = run.result()
    assert status & L.ST_BAD_INDEX and np.all(out.view(np.uint8) == 0xCD)
    # host-visible errors
    run = hip.MatRun(mp, want_dims=False)
    assert fdy.fdy_materialize(run.desc, run.d_out, None, run.d_ws, run.ws_bytes - 1, run.d_status,
                               check=False) == fdy.FDY_ERR_WORKSPACE
    assert fdy.fdy_materialize(run.desc, run.d_out.data_ptr() + 8, None, run.d_ws, run.ws_bytes,
                               run.d_status, check=False) == fdy.FDY_ERR_INVALID_ARG


def test_materialize_lists_out_of_order_are_flagged(hip, oracle):
    """Every list must ascend strictly by location (the tile slices are found by binary search):
    a swapped pair, or a location twice, in a relocation, override, grid-override or patch list
    raises FDY_ST_BAD_ORDER on the device, at the start, in the middle and across a tile edge;
    the oracle refuses the same inputs.  Valid inputs raise nothing."""
    rng = np.random.default_rng(11)
    for idx in (2, 3):
        ar = small(idx)
        mp = problem(oracle, ar, maps=[0, 1] if idx == 3 else None)
        base = {n: getattr(mp, n) for n in MatProblem.ARRAYS}
        _, _, status = hip.materialize(MatProblem(n_ranks=mp.n_ranks, **base))
        assert status == 0

        def damaged(name, off_name, key, rows, how):
            """One list of kind `name` (a row of its offset array that has at least 3 entries)
            with entries i, i+1 swapped or made equal."""
            arr = getattr(mp, name).copy()
            off = getattr(mp, off_name).astype(np.int64)
            rows = [r for r in rows if off[r + 1] - off[r] >= 3]
            r = rows[int(rng.integers(len(rows)))]
            n = off[r + 1] - off[r]
            for where in (0, n // 2, n - 2):
                a = arr.copy()
                i = off[r] + where
                if how == "swap":
                    a[[i, i + 1]] = a[[i + 1, i]]
                else:
                    a[key][i + 1] = a[key][i]
                yield a

        kinds = [("relocs", "src_reloc_off", "word", [int(s) for s in mp.tmpl_graph]),
                 ("ovr", "ovr_off", "byte_off", range(mp.G)),
                 ("govr", "govr_off", "node", range(mp.G))]
        if mp.map_rank is not None:
            kinds.append(("patch", "patch_off", "word", range(mp.T * mp.n_ranks)))
        for name, off_name, key, rows in kinds:
            for how in ("swap", "equal"):
                for arr in damaged(name, off_name, key, list(rows), how):
                    kw = dict(base)
                    kw[name] = arr
                    bad = MatProblem(n_ranks=mp.n_ranks, **kw)
                    say(f"[order] config {idx}: {name} {how}")
                    with pytest.raises(Exception):
                        oracle.materialize(bad)
                    _, _, status = hip.materialize(bad)
                    assert status & L.ST_BAD_ORDER, (name, how, status)
    # a long relocation list whose disorder sits exactly at a tile edge (words 2047 | 2048)
    ar = small(4)
    mp = problem(oracle, ar)
    rel = mp.relocs.copy()
    i = int(np.searchsorted(rel["word"], 2048))
    assert 0 < i < len(rel) - 1
    rel[[i - 1, i]] = rel[[i, i - 1]]
    kw = {n: getattr(mp, n) for n in MatProblem.ARRAYS}
    kw["relocs"] = rel
    _, _, status = hip.materialize(MatProblem(n_ranks=0, **kw), want_dims=False)
    assert status & L.ST_BAD_ORDER


# ------------------------------------------------------------------- whole path, full sizes
@pytest.mark.parametrize("idx", [1, 2, 3, 5, 4])
def test_full_config_whole_path(hip, oracle, idx):
    """The whole path chained on the device (no host round trip between the calls), at the full
    size of each configuration, every output compared with the oracle element by element.
    Twice: in the launch configuration that bench.py times (table prepared once, segmentation
    and fingerprint in one launch, and - where every graph is its own template under one base
    map, config 4 - the scan writing the materialized output itself), and through the plain
    calls (fdy_scan_pointers, fdy_reloc_segment, fdy_fingerprint, fdy_materialize)."""
    import paper_2604_06664_amd as fdy
    import torch

    say(f"[full] config {idx}: generating")
    ar = make_config(idx)
    say(f"[full] config {idx}: oracle")
    relocs, cnt = oracle.scan(ar.words, ar.table)
    roff = oracle.reloc_segment(relocs, ar.word_off)
    keys, tid, tg = oracle.fingerprint(ar.nodes, ar.node_off, ar.fp_mask)
    assert np.array_equal(tid, ar.graph_tmpl) and np.array_equal(tg, ar.tmpl_graph)
    mp = MatProblem.from_archive(ar, relocs, roff, graph_tmpl=tid, tmpl_graph=tg)
    want_dims = len(ar.nodes) > 0
    ref, rdims = oracle.materialize(mp, want_dims=want_dims)
    G = ar.n_graphs
    for how in ("as benchmarked", "plain calls"):
        bench_like = how == "as benchmarked"
        say(f"[full] config {idx}: gpu, {how}: W={len(ar.words)} A={ar.n_alloc} G={G} M={ar.n_maps}")
        run = hip.PathRun(ar, reloc_capacity=cnt + 16, prepared=bench_like, one_pass=None if bench_like else False)
        assert run.one_pass == (bench_like and idx == 4)
        for t in (run.scan.d_relocs, run.mat.d_out):
            t.fill_(0xEE)
        run.step()
        assert run.status() == 0
        got_cnt = int(run.scan.d_count.item())
        assert got_cnt == cnt == len(ar.ptr_word)
        say(f"[full] config {idx}: comparing")
        assert np.array_equal(fdy.to_host(run.scan.d_relocs, hip.RELOC, cnt), relocs)
        assert np.array_equal(fdy.to_host(run.d_reloc_off, np.uint64, G + 1), roff)
        nt = int(run.d_nt.item())
        assert nt == len(tg)
        assert np.array_equal(fdy.to_host(run.d_keys, np.uint64, G), keys)
        assert np.array_equal(fdy.to_host(run.d_tid, np.uint32, G), tid)
        assert np.array_equal(fdy.to_host(run.d_tg, np.uint32, nt), tg)
        out = fdy.to_host(run.mat.d_out, np.uint64, mp.M * run.mat.wpm).reshape(mp.M, run.mat.wpm)
        assert np.array_equal(out, ref)
        del out
        if rdims is not None:
            assert np.array_equal(fdy.to_host(run.mat.d_dims, np.uint32, run.mat.nodes_total * 6).reshape(-1, 6), rdims)
        del run
        torch.cuda.empty_cache()


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_repeated_runs_give_identical_bytes(hip, idx):
    """Workgroups draw their chunks in whatever order they start, and hits are placed by a
    look-back over other workgroups' totals: a race there would show as outputs that differ
    from run to run.  The whole path runs four times over poisoned outputs and workspaces,
    with an unrelated kernel in between; every byte of every output must repeat.  (Each
    configuration's outputs are compared with the oracle in test_full_config_whole_path.)"""
    import torch

    ar = make_config(idx)
    say(f"[repeat] config {idx}: W={len(ar.words)} A={ar.n_alloc}")
    run = hip.PathRun(ar, reloc_capacity=len(ar.ptr_word) + 16)
    outs = [run.scan.d_relocs, run.scan.d_count, run.d_reloc_off, run.d_keys, run.d_tid, run.d_tg, run.d_nt,
            run.mat.d_out] + ([run.mat.d_dims] if run.mat.d_dims is not None else [])
    first = None
    for rep in range(4):
        # outputs and workspaces are poisoned; the prepared table is not (its counters must have
        # been left zeroed by the run before)
        for t in outs + [run.scan.d_ws, run.mat.d_ws]:
            t.fill_(0x5A + rep)
        run.step()
        assert run.status() == 0
        n = int(run.scan.d_count.item())
        assert n == len(ar.ptr_word)
        n_tmpl = int(run.d_nt.item())  # only that many entries of the template list are written
        cut = {id(run.scan.d_relocs): n * 16, id(run.d_tg): n_tmpl * 4}
        got = [t[: cut[id(t)]].clone() if id(t) in cut else t.clone() for t in outs]
        if first is None:
            first = got
        else:
            for a, b in zip(first, got):
                assert torch.equal(a, b)
        torch.rand(1 << 20, device="cuda").sum().item()  # something else on the device in between
    del run, first, got
    torch.cuda.empty_cache()
