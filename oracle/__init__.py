"""ctypes binding of the CPU oracle (oracle/fdy_oracle.cpp).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the bench's cpu_baseline leg may
import this package; the product package never does.  Every function takes and returns
numpy arrays in host memory.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

from synth import layout as L
from synth.problem import MatProblem

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "fdy_oracle.cpp")
# FDY_ORACLE_LIB: load this prebuilt library instead (the mutation test points it at copies of
# the oracle with a planted mistake, to show that the pins notice)
_ALT = os.environ.get("FDY_ORACLE_LIB")
_LIB = _ALT or os.path.join(_DIR, "libfdy_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with the host compiler (no GPU toolchain involved)."""
    if _ALT:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["g++", "-std=c++17", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", _SRC, "-o", _LIB])
    return _LIB


class _MatArgs(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("S", "T", "G", "M", "A", "R")] + [
        (n, C.c_void_p)
        for n in ("src_words", "src_word_off", "src_nodes", "src_node_off", "relocs",
                  "src_reloc_off", "tmpl_graph", "graph_tmpl", "ovr", "ovr_off", "govr",
                  "govr_off", "new_base", "map_rank", "patch", "patch_off")
    ]


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.orc_mix.restype = C.c_uint64
        _lib.orc_mix.argtypes = [C.c_uint64]
    return _lib


def _p(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def mix(x: int) -> int:
    return int(lib().orc_mix(C.c_uint64(x & (2**64 - 1))))


def table_validate(table):
    t = _c(table, L.ALLOC)
    bad = C.c_uint32(0xFFFFFFFF)
    rc = lib().orc_table_validate(_p(t), C.c_uint32(len(t)), C.byref(bad))
    return rc, bad.value


def layout_invert(table, new_base):
    """Inverse of a base map: the new layout as a table sorted by new base, the captured bases
    in that order, and which captured region each entry is.  Returns None if regions overlap
    or wrap at their new places (plain Python integers; definition written out)."""
    t = _c(table, L.ALLOC)
    placed = sorted((int(nb), int(sz), int(ob), r)
                    for r, (nb, sz, ob) in enumerate(zip(new_base, t["size"], t["base"])))
    for k, (nb, sz, _, _) in enumerate(placed):
        if sz < 1 or nb + sz >= 1 << 64 or (k and nb < placed[k - 1][0] + placed[k - 1][1]):
            return None
    inv = np.zeros(len(placed), L.ALLOC)
    inv["base"] = [p[0] for p in placed]
    inv["size"] = [p[1] for p in placed]
    return inv, np.array([p[2] for p in placed], np.uint64), np.array([p[3] for p in placed], np.uint32)


def layout_replay(recorded, recorded_start, new_start, new_capacity, new_used=0):
    """A recorded layout placed in a new address range (Section 4.1.1 capture-window replay,
    Section 5.1): every allocation keeps its distance from the start of the range.  Returns the
    new bases, or the name of what is wrong ("table", "order", "capacity").  Plain Python
    integers; definition written out."""
    t = _c(recorded, L.ALLOC)
    rows = [(int(b), int(z)) for b, z in zip(t["base"], t["size"])]
    if not rows:
        return np.zeros(0, np.uint64)
    for k, (b, z) in enumerate(rows):
        if z < 1 or b + z > (1 << 64) - 1 or (k and b < rows[k - 1][0] + rows[k - 1][1]):
            return "table"
    if rows[0][0] < recorded_start:
        return "table"
    dist = [b - recorded_start for b, _ in rows]
    if dist[0] < new_used:
        return "order"
    end = dist[-1] + rows[-1][1]
    if end > new_capacity or new_start + end > (1 << 64) - 1:  # the placed table must be valid too
        return "capacity"
    return np.array([new_start + d for d in dist], np.uint64)


def _scan(fn, words, table, capacity=None):
    w = _c(words, np.uint64)
    t = _c(table, L.ALLOC)
    cap = len(w) if capacity is None else int(capacity)
    out = np.zeros(cap, L.RELOC)
    cnt = C.c_uint64(0)
    rc = fn(_p(w), C.c_uint64(len(w)), _p(t), C.c_uint32(len(t)), _p(out), C.c_uint64(cap),
            C.byref(cnt))
    assert rc == 0
    return out[: min(cnt.value, cap)].copy(), cnt.value


def scan(words, table, capacity=None):
    """-> (relocs RELOC[min(count,capacity)], count)"""
    return _scan(lib().orc_scan, words, table, capacity)


def scan_brute(words, table, capacity=None):
    return _scan(lib().orc_scan_brute, words, table, capacity)


def scan_stride4(units, table, capacity=None):
    """units: uint32 array.  -> (relocs RELOC[min(count,capacity)] with word = position, count)"""
    u = _c(units, np.uint32)
    t = _c(table, L.ALLOC)
    cap = max(len(u) - 1, 0) if capacity is None else int(capacity)
    out = np.zeros(cap, L.RELOC)
    cnt = C.c_uint64(0)
    rc = lib().orc_scan_stride4(_p(u), C.c_uint64(len(u)), _p(t), C.c_uint32(len(t)), _p(out), C.c_uint64(cap),
                                C.byref(cnt))
    assert rc == 0
    return out[: min(cnt.value, cap)].copy(), cnt.value


def reloc_segment(relocs, word_off):
    r = _c(relocs, L.RELOC)
    wo = _c(word_off, np.uint64)
    out = np.zeros(len(wo), np.uint64)
    rc = lib().orc_reloc_segment(_p(r), C.c_uint64(len(r)), _p(wo), C.c_uint32(len(wo)), _p(out))
    assert rc == 0
    return out


def fingerprint(nodes, node_off, mask):
    """-> (keys u64[G], template_id u32[G], tmpl_graph u32[T])"""
    n = _c(nodes, L.NODE)
    no = _c(node_off, np.uint64)
    G = len(no) - 1
    keys = np.zeros(G, np.uint64)
    tid = np.zeros(G, np.uint32)
    tg = np.zeros(G, np.uint32)
    nt = C.c_uint32(0)
    rc = lib().orc_fingerprint(_p(n), _p(no), C.c_uint32(G), C.c_uint32(mask), _p(keys), _p(tid),
                               _p(tg), C.byref(nt))
    assert rc == 0
    return keys, tid, tg[: nt.value].copy()


def fingerprint_powersum(nodes, node_off, mask):
    n = _c(nodes, L.NODE)
    no = _c(node_off, np.uint64)
    G = len(no) - 1
    keys = np.zeros(G, np.uint64)
    rc = lib().orc_fingerprint_powersum(_p(n), _p(no), C.c_uint32(G), C.c_uint32(mask), _p(keys))
    assert rc == 0
    return keys


def group_exact(nodes, node_off, mask):
    n = _c(nodes, L.NODE)
    no = _c(node_off, np.uint64)
    G = len(no) - 1
    tid = np.zeros(G, np.uint32)
    tg = np.zeros(G, np.uint32)
    nt = C.c_uint32(0)
    rc = lib().orc_group_exact(_p(n), _p(no), C.c_uint32(G), C.c_uint32(mask), _p(tid), _p(tg),
                               C.byref(nt))
    assert rc == 0
    return tid, tg[: nt.value].copy()


def _mat_args(mi: MatProblem):
    a = _MatArgs()
    a.S, a.T, a.G, a.M, a.A, a.R = mi.S, mi.T, mi.G, mi.M, mi.A, mi.n_ranks
    for n in MatProblem.ARRAYS:
        v = getattr(mi, n)
        setattr(a, n, None if v is None else v.ctypes.data)
    return a


def materialize_validate(mi: MatProblem):
    a = _mat_args(mi)
    return lib().orc_materialize_validate(C.byref(a), C.c_uint64(mi.out_words_per_map()),
                                          C.c_uint64(mi.out_nodes_total()))


def materialize(mi: MatProblem, want_dims=True):
    """-> (out_words u64[M][out_words_per_map], out_dims u32[out_nodes_total][6] | None)"""
    a = _mat_args(mi)
    wpm, nt = mi.out_words_per_map(), mi.out_nodes_total()
    out = np.zeros((mi.M, wpm), np.uint64)
    dims = np.zeros((nt, 6), np.uint32) if want_dims else None
    rc = lib().orc_materialize(C.byref(a), _p(out), C.c_uint64(wpm), _p(dims), C.c_uint64(nt))
    if rc != 0:
        raise ValueError("oracle: materialize inputs are not valid")
    return out, dims


def materialize_brute(mi: MatProblem):
    a = _mat_args(mi)
    wpm = mi.out_words_per_map()
    out = np.zeros((mi.M, wpm), np.uint64)
    rc = lib().orc_materialize_brute(C.byref(a), _p(out), C.c_uint64(wpm))
    if rc != 0:
        raise ValueError("oracle: materialize inputs are not valid")
    return out


def derive_overrides(words, word_off, graph_tmpl, tmpl_graph, capacity=None):
    """-> (ovr OVR32[min(total, capacity)], ovr_off u64[G+1]); raises on mismatched sizes."""
    w = _c(words, np.uint64)
    wo = _c(word_off, np.uint64)
    gt = _c(graph_tmpl, np.uint32)
    tg = _c(tmpl_graph, np.uint32)
    G = len(gt)
    cap = 2 * len(w) if capacity is None else int(capacity)
    ovr = np.zeros(cap, L.OVR32)
    off = np.zeros(G + 1, np.uint64)
    rc = lib().orc_derive_overrides(_p(w), _p(wo), C.c_uint32(G), _p(gt), _p(tg), C.c_uint32(len(tg)),
                                    _p(ovr), C.c_uint64(cap), _p(off))
    if rc != 0:
        raise ValueError("oracle: derive_overrides inputs are not valid")
    return ovr[: min(int(off[G]), cap)].copy(), off
