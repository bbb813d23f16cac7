"""Host-only checks of the C-ABI library: it loads, exports every symbol the public header
declares, and its host-side logic (table validation, workspace sizing, argument checks that
return before any GPU call) behaves.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from synth import layout as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def fdy():
    import paper_2604_06664_amd as m

    if not os.path.exists(m.LIB_PATH):
        from paper_2604_06664_amd.build import build_lib

        build_lib()
    m.lib()
    return m


def declared_functions():
    """Every function declared by a header under include/."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for h in sorted(os.listdir(inc)):
        if h.endswith(".h"):
            src = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, h)).read(), flags=re.S)
            names |= set(re.findall(r"\b(fdy_[a-z_0-9]+)\s*\(", src))
    return sorted(names)


def test_every_declared_symbol_is_exported(fdy):
    names = declared_functions()
    assert {"fdy_scan_pointers", "fdy_fingerprint", "fdy_materialize", "fdy_reloc_segment",
            "fdy_table_validate", "fdy_scan_workspace_bytes", "fdy_materialize_workspace_bytes",
            "fdy_version", "fdy_strerror", "fdy_scan_rebase", "fdy_derive_overrides",
            "fdy_derive_workspace_bytes", "fdy_arena_create", "fdy_arena_alloc", "fdy_arena_table",
            "fdy_arena_destroy", "fdy_arena_replay", "fdy_layout_replay", "fdy_layout_invert"} <= set(names)
    raw = C.CDLL(fdy.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), f"{n} declared in fdy.h but not exported"


def test_version_and_error_strings(fdy):
    assert fdy.fdy_version() == 300
    for code in range(0, -7, -1):
        assert fdy.fdy_strerror(code) not in ("", "unknown fdy error code")
    assert fdy.fdy_strerror(-99) == "unknown fdy error code"


def test_struct_sizes_match_header(fdy):
    assert C.sizeof(fdy.fdy_mat_desc) == 6 * 4 + 2 * 8 + 16 * 8


def mk(pairs):
    t = np.zeros(len(pairs), L.ALLOC)
    for i, p in enumerate(pairs):
        t[i] = p
    return t


def test_table_validate_agrees_with_oracle(fdy, oracle):
    cases = [
        [(10, 5), (15, 5), (30, 1)], [(10, 5), (14, 5)], [(10, 5), (10, 5)], [(10, 0)],
        [(2**64 - 4, 4)], [(2**64 - 4, 3)], [(30, 1), (10, 5)], [], [(0, 1)], [(5, 2**64 - 6), (2**64 - 1, 1)],
    ]
    rng = np.random.default_rng(1)
    for _ in range(200):
        n = int(rng.integers(1, 6))
        cases.append([(int(b), int(s)) for b, s in zip(np.sort(rng.integers(0, 60, n)), rng.integers(0, 12, n))])
    for c in cases:
        t = mk(c)
        rc, bad = fdy.fdy_table_validate(t)
        orc, obad = oracle.table_validate(t)
        assert (rc == 0) == (orc == 0), c
        if rc != 0:
            assert rc == fdy.FDY_ERR_TABLE and bad == obad, c


def test_workspace_sizes(fdy):
    assert fdy.fdy_scan_workspace_bytes(0, 0) >= 256
    a = fdy.fdy_scan_workspace_bytes(1 << 27, 1 << 20)
    # table hierarchy (about 14 MiB for 2^20 allocations) and chunk states; the staging area of
    # dense inputs is optional, queried apart, and bounded by the workgroups in flight (160 MiB)
    assert 0 < a < 32 << 20 and a % 256 == 0
    assert 0 < fdy.fdy_scan_staging_bytes(1 << 27) <= 160 << 20
    assert fdy.fdy_scan_staging_bytes(1 << 31) == fdy.fdy_scan_staging_bytes(1 << 27)
    assert fdy.fdy_scan_workspace_bytes(1 << 31, 1 << 20) - a < 8 << 20  # 16 times the words: chunk states only
    assert fdy.fdy_scan_workspace_bytes(1 << 17, 256) + fdy.fdy_scan_staging_bytes(1 << 17) < 8 << 20
    t = fdy.fdy_scan_table_bytes(1 << 20, 1 << 27)
    assert 0 < t < 32 << 20 and t % 256 == 0 and fdy.fdy_scan_table_bytes(16, 1 << 32) == 0
    assert fdy.fdy_fingerprint_workspace_bytes(67) == 256 and fdy.fdy_fingerprint_workspace_bytes((1 << 20) + 1) == 0
    assert fdy.fdy_fingerprint_workspace_bytes(1 << 20) == 8 << 20
    assert fdy.fdy_scan_workspace_bytes(1 << 32, 16) == 0  # word index must fit 32 bits
    d = fdy.fdy_mat_desc()
    d.n_graphs, d.n_maps, d.out_words_per_map = 67, 256, 761364
    w = fdy.fdy_materialize_workspace_bytes(d)
    assert 0 < w < 1 << 20 and w % 256 == 0
    d.n_maps = 70000
    assert fdy.fdy_materialize_workspace_bytes(d) == 0


def test_argument_checks_that_need_no_gpu(fdy):
    # all of these return before any HIP call is made
    assert fdy.lib().fdy_scan_pointers(None, 8, None, 0, None, 0, None, None, None, 0, None, None) == fdy.FDY_ERR_INVALID_ARG
    assert fdy.lib().fdy_fingerprint(None, None, (1 << 20) + 1, L.FP_ALL, None, None, None, None, None, 0, None) == fdy.FDY_ERR_INVALID_ARG
    assert fdy.lib().fdy_fingerprint(None, None, 1, 0x80, None, None, None, None, None, 0, None) == fdy.FDY_ERR_INVALID_ARG
    d = fdy.fdy_mat_desc()
    d.n_graphs, d.n_maps = 1, 1
    assert fdy.lib().fdy_materialize(C.byref(d), None, None, None, 0, None, None) == fdy.FDY_ERR_INVALID_ARG
    assert fdy.tune_set(99, 1) == -1 and fdy.tune_set(fdy.TUNE_SCAN_TOP_LOG2, 40) == -1
