"""paper_2604_06664_amd - thin Python binding of libfdy (the HIP/gfx950 C-ABI library).

Argument marshalling only: every step of the path runs in the library's kernels.  PyTorch
supplies device memory and streams.  There is no CPU fallback: if the built library is
missing, importing the binding functions raises.

Entry points keep the names of include/fdy.h: fdy_scan_pointers, fdy_scan_pointers_stride4, fdy_scan_rebase,
fdy_scan_pointers_rebase,
fdy_reloc_segment, fdy_fingerprint, fdy_derive_overrides, fdy_materialize (+ workspace queries,
fdy_table_validate, fdy_layout_invert, fdy_layout_replay, fdy_strerror); include/fdy_archive.h is bound in archive.py.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfdy.so")
_lib = None

FDY_OK = 0
FDY_ERR_INVALID_ARG, FDY_ERR_TABLE, FDY_ERR_CAPACITY = -1, -2, -3
FDY_ERR_HIP, FDY_ERR_WORKSPACE, FDY_ERR_ORDER = -4, -5, -6

TUNE_SCAN_TOP_LOG2, TUNE_SCAN_WG_PER_CU, TUNE_SCAN_SPIN_LIMIT, TUNE_MAT_MAP_GROUP = 0, 1, 2, 3
TUNE_SCAN_SMALL_LOG2 = 4
TUNE_MAT_SELF_WGS = 5
TUNE_MAT_ONCE_TILES = 6


class FdyError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {fdy_strerror(code)} ({code})")


class fdy_mat_desc(C.Structure):
    _fields_ = (
        [(n, C.c_uint32) for n in ("n_src_graphs", "n_templates", "n_graphs", "n_maps", "n_alloc", "n_ranks")]
        + [("out_words_per_map", C.c_uint64), ("out_nodes_total", C.c_uint64)]
        + [(n, C.c_void_p) for n in ("src_words", "src_word_off", "src_nodes", "src_node_off", "relocs",
                                      "src_reloc_off", "tmpl_graph", "graph_tmpl", "ovr", "ovr_off",
                                      "govr", "govr_off", "new_base", "map_rank", "patch", "patch_off")]
    )


def lib():
    """The loaded C-ABI library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2604_06664_amd.build` "
                "(hipcc, gfx950). There is no CPU fallback.")
        L = C.CDLL(LIB_PATH)
        L.fdy_version.restype = C.c_int
        L.fdy_strerror.restype = C.c_char_p
        L.fdy_strerror.argtypes = [C.c_int]
        L.fdy_table_validate.restype = C.c_int
        L.fdy_table_validate.argtypes = [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint32)]
        L.fdy_layout_invert.restype = C.c_int
        L.fdy_layout_invert.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.fdy_layout_replay.restype = C.c_int
        L.fdy_layout_replay.argtypes = [C.c_void_p, C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64,
                                        C.c_void_p]
        L.fdy_scan_workspace_bytes.restype = C.c_size_t
        L.fdy_scan_workspace_bytes.argtypes = [C.c_uint64, C.c_uint32]
        L.fdy_scan_staging_bytes.restype = C.c_size_t
        L.fdy_scan_staging_bytes.argtypes = [C.c_uint64]
        L.fdy_scan_pointers.restype = C.c_int
        L.fdy_scan_pointers.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p,
                                        C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                        C.c_void_p, C.c_void_p]
        L.fdy_scan_table_bytes.restype = C.c_size_t
        L.fdy_scan_table_bytes.argtypes = [C.c_uint32, C.c_uint64]
        L.fdy_scan_table_prepare.restype = C.c_int
        L.fdy_scan_table_prepare.argtypes = [C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p, C.c_size_t,
                                             C.c_void_p]
        L.fdy_scan_pointers_stride4.restype = C.c_int
        L.fdy_scan_pointers_stride4.argtypes = L.fdy_scan_pointers.argtypes
        L.fdy_scan_rebase.restype = C.c_int
        L.fdy_scan_rebase.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                      C.c_void_p, C.c_void_p]
        L.fdy_scan_pointers_rebase.restype = C.c_int
        L.fdy_scan_pointers_rebase.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p,
                                               C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.fdy_reloc_segment.restype = C.c_int
        L.fdy_reloc_segment.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32,
                                        C.c_void_p, C.c_void_p]
        L.fdy_fingerprint.restype = C.c_int
        L.fdy_fingerprint.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.fdy_fingerprint_workspace_bytes.restype = C.c_size_t
        L.fdy_fingerprint_workspace_bytes.argtypes = [C.c_uint32]
        L.fdy_segment_fingerprint.restype = C.c_int
        L.fdy_segment_fingerprint.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_size_t, C.c_void_p]
        L.fdy_derive_workspace_bytes.restype = C.c_size_t
        L.fdy_derive_workspace_bytes.argtypes = [C.c_uint64, C.c_uint32]
        L.fdy_derive_overrides.restype = C.c_int
        L.fdy_derive_overrides.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p,
                                           C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint64, C.c_void_p,
                                           C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.fdy_materialize_workspace_bytes.restype = C.c_size_t
        L.fdy_materialize_workspace_bytes.argtypes = [C.POINTER(fdy_mat_desc)]
        L.fdy_materialize.restype = C.c_int
        L.fdy_materialize.argtypes = [C.POINTER(fdy_mat_desc), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_size_t, C.c_void_p, C.c_void_p]
        L.fdy_materialize_static_limit.restype = C.c_size_t
        L.fdy_materialize_static_limit.argtypes = []
        L.fdy_materialize_static.restype = C.c_int
        L.fdy_materialize_static.argtypes = [C.POINTER(fdy_mat_desc), C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p]
        L.fdy__tune_get.restype = C.c_int
        L.fdy__tune_get.argtypes = [C.c_int]
        L.fdy__tune_set.restype = C.c_int
        L.fdy__tune_set.argtypes = [C.c_int, C.c_int]
        L.fdy__prof_enable.restype = C.c_int
        L.fdy__prof_enable.argtypes = [C.c_int]
        L.fdy__prof_mask.restype = None
        L.fdy__prof_mask.argtypes = [C.c_uint]
        L.fdy__prof_read.restype = C.c_int
        L.fdy__prof_read.argtypes = [C.c_int, C.POINTER(C.c_int)] + [C.POINTER(C.c_float)] * 3
        L.fdy__prof_name.restype = C.c_char_p
        L.fdy__prof_name.argtypes = [C.c_int]
        _lib = L
    return _lib


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch

        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _check(rc, where):
    if rc != FDY_OK:
        raise FdyError(rc, where)
    return rc


# ---- entry points (names as in include/fdy.h) --------------------------------------------
def fdy_version():
    return lib().fdy_version()


def fdy_strerror(code):
    return lib().fdy_strerror(int(code)).decode()


def fdy_table_validate(h_table):
    """h_table: numpy array of fdy_alloc records in host memory -> (rc, bad_index)."""
    t = np.ascontiguousarray(h_table)
    assert t.dtype.itemsize == 16
    bad = C.c_uint32(0xFFFFFFFF)
    rc = lib().fdy_table_validate(t.ctypes.data if len(t) else None, len(t), C.byref(bad))
    return rc, bad.value


def fdy_layout_invert(h_table, h_new_base, check=True):
    """h_table: fdy_alloc records, h_new_base: uint64 per region (host numpy arrays) ->
    (rc, inv_table, inv_base, inv_region) as new host arrays."""
    t = np.ascontiguousarray(h_table)
    nb = np.ascontiguousarray(h_new_base, np.uint64)
    assert t.dtype.itemsize == 16 and len(nb) == len(t)
    inv_t, inv_b, inv_r = np.zeros_like(t), np.zeros(len(t), np.uint64), np.zeros(len(t), np.uint32)
    rc = lib().fdy_layout_invert(_ptr(t) if len(t) else None, _ptr(nb) if len(t) else None, len(t),
                                 _ptr(inv_t) if len(t) else None, _ptr(inv_b) if len(t) else None,
                                 _ptr(inv_r) if len(t) else None)
    if check:
        _check(rc, "fdy_layout_invert")
    return rc, inv_t, inv_b, inv_r


def fdy_layout_replay(h_recorded, recorded_start, new_start, new_capacity, new_used=0, check=True):
    """h_recorded: fdy_alloc records (host numpy array) -> (rc, new_base uint64 per allocation)."""
    t = np.ascontiguousarray(h_recorded)
    assert t.dtype.itemsize == 16
    nb = np.zeros(len(t), np.uint64)
    rc = lib().fdy_layout_replay(_ptr(t) if len(t) else None, len(t), int(recorded_start), int(new_start),
                                 int(new_capacity), int(new_used), _ptr(nb) if len(t) else None)
    if check:
        _check(rc, "fdy_layout_replay")
    return rc, nb


def fdy_scan_workspace_bytes(n_words, n_alloc):
    return lib().fdy_scan_workspace_bytes(int(n_words), int(n_alloc))


def fdy_scan_staging_bytes(n_words):
    return lib().fdy_scan_staging_bytes(int(n_words))


def fdy_scan_table_bytes(n_alloc, max_words):
    return lib().fdy_scan_table_bytes(int(n_alloc), int(max_words))


def fdy_scan_table_prepare(d_table, n_alloc, max_words, d_prepared, prepared_bytes, stream=None,
                           check=True):
    rc = lib().fdy_scan_table_prepare(_ptr(d_table), int(n_alloc), int(max_words), _ptr(d_prepared),
                                      int(prepared_bytes), _stream(stream))
    return _check(rc, "fdy_scan_table_prepare") if check else rc


def fdy_scan_pointers(d_words, n_words, d_table, n_alloc, d_relocs, reloc_capacity, d_count,
                      d_prepared, d_workspace, workspace_bytes, d_status=None, stream=None, check=True):
    rc = lib().fdy_scan_pointers(_ptr(d_words), int(n_words), _ptr(d_table), int(n_alloc),
                                 _ptr(d_relocs), int(reloc_capacity), _ptr(d_count), _ptr(d_prepared),
                                 _ptr(d_workspace), int(workspace_bytes), _ptr(d_status),
                                 _stream(stream))
    return _check(rc, "fdy_scan_pointers") if check else rc


def fdy_scan_pointers_stride4(d_units, n_units, d_table, n_alloc, d_relocs, reloc_capacity, d_count,
                              d_prepared, d_workspace, workspace_bytes, d_status=None, stream=None,
                              check=True):
    rc = lib().fdy_scan_pointers_stride4(_ptr(d_units), int(n_units), _ptr(d_table), int(n_alloc),
                                         _ptr(d_relocs), int(reloc_capacity), _ptr(d_count),
                                         _ptr(d_prepared), _ptr(d_workspace), int(workspace_bytes),
                                         _ptr(d_status), _stream(stream))
    return _check(rc, "fdy_scan_pointers_stride4") if check else rc


def fdy_scan_rebase(d_words, n_words, d_table, n_alloc, d_new_base, d_out_words, d_count,
                    d_prepared, d_workspace, workspace_bytes, d_status=None, stream=None, check=True):
    rc = lib().fdy_scan_rebase(_ptr(d_words), int(n_words), _ptr(d_table), int(n_alloc),
                               _ptr(d_new_base), _ptr(d_out_words), _ptr(d_count), _ptr(d_prepared),
                               _ptr(d_workspace), int(workspace_bytes), _ptr(d_status), _stream(stream))
    return _check(rc, "fdy_scan_rebase") if check else rc


def fdy_scan_pointers_rebase(d_words, n_words, d_table, n_alloc, d_relocs, reloc_capacity, d_count,
                             d_new_base, d_out_words, d_prepared, d_workspace, workspace_bytes,
                             d_status=None, stream=None, check=True):
    rc = lib().fdy_scan_pointers_rebase(_ptr(d_words), int(n_words), _ptr(d_table), int(n_alloc),
                                        _ptr(d_relocs), int(reloc_capacity), _ptr(d_count),
                                        _ptr(d_new_base), _ptr(d_out_words), _ptr(d_prepared),
                                        _ptr(d_workspace), int(workspace_bytes), _ptr(d_status),
                                        _stream(stream))
    return _check(rc, "fdy_scan_pointers_rebase") if check else rc


def fdy_reloc_segment(d_relocs, d_count, reloc_capacity, d_word_off, n_off, d_reloc_off,
                      stream=None, check=True):
    rc = lib().fdy_reloc_segment(_ptr(d_relocs), _ptr(d_count), int(reloc_capacity),
                                 _ptr(d_word_off), int(n_off), _ptr(d_reloc_off), _stream(stream))
    return _check(rc, "fdy_reloc_segment") if check else rc


def fdy_fingerprint_workspace_bytes(n_graphs):
    return lib().fdy_fingerprint_workspace_bytes(int(n_graphs))


def fdy_fingerprint(d_nodes, d_node_off, n_graphs, field_mask, d_keys, d_template_id, d_tmpl_graph,
                    d_n_templates, stream=None, check=True, d_workspace=None, workspace_bytes=0):
    rc = lib().fdy_fingerprint(_ptr(d_nodes), _ptr(d_node_off), int(n_graphs), int(field_mask),
                               _ptr(d_keys), _ptr(d_template_id), _ptr(d_tmpl_graph),
                               _ptr(d_n_templates), _ptr(d_workspace), int(workspace_bytes), _stream(stream))
    return _check(rc, "fdy_fingerprint") if check else rc


def fdy_segment_fingerprint(d_relocs, d_count, reloc_capacity, d_word_off, d_reloc_off, d_nodes, d_node_off,
                            n_graphs, field_mask, d_keys, d_template_id, d_tmpl_graph, d_n_templates,
                            d_prepared=None, d_workspace=None, workspace_bytes=0, stream=None, check=True):
    rc = lib().fdy_segment_fingerprint(_ptr(d_relocs), _ptr(d_count), int(reloc_capacity), _ptr(d_word_off),
                                       _ptr(d_reloc_off), _ptr(d_nodes), _ptr(d_node_off), int(n_graphs),
                                       int(field_mask), _ptr(d_keys), _ptr(d_template_id), _ptr(d_tmpl_graph),
                                       _ptr(d_n_templates), _ptr(d_prepared), _ptr(d_workspace),
                                       int(workspace_bytes), _stream(stream))
    return _check(rc, "fdy_segment_fingerprint") if check else rc


def fdy_derive_workspace_bytes(n_words_total, n_graphs):
    return lib().fdy_derive_workspace_bytes(int(n_words_total), int(n_graphs))


def fdy_derive_overrides(d_words, n_words_total, d_word_off, n_graphs, d_graph_tmpl, d_tmpl_graph,
                         n_templates, d_ovr, ovr_capacity, d_ovr_off, d_workspace, workspace_bytes,
                         d_status=None, stream=None, check=True):
    rc = lib().fdy_derive_overrides(_ptr(d_words), int(n_words_total), _ptr(d_word_off), int(n_graphs),
                                    _ptr(d_graph_tmpl), _ptr(d_tmpl_graph), int(n_templates),
                                    _ptr(d_ovr), int(ovr_capacity), _ptr(d_ovr_off), _ptr(d_workspace),
                                    int(workspace_bytes), _ptr(d_status), _stream(stream))
    return _check(rc, "fdy_derive_overrides") if check else rc


def fdy_materialize_workspace_bytes(h_desc):
    return lib().fdy_materialize_workspace_bytes(C.byref(h_desc))


def fdy_materialize(h_desc, d_out_words, d_out_dims, d_workspace, workspace_bytes, d_status=None,
                    stream=None, check=True):
    rc = lib().fdy_materialize(C.byref(h_desc), _ptr(d_out_words), _ptr(d_out_dims),
                               _ptr(d_workspace), int(workspace_bytes), _ptr(d_status),
                               _stream(stream))
    return _check(rc, "fdy_materialize") if check else rc


def fdy_materialize_static_limit():
    return lib().fdy_materialize_static_limit()


def fdy_materialize_static(h_desc, d_out_words, d_out_dims, d_status=None, stream=None, check=True):
    rc = lib().fdy_materialize_static(C.byref(h_desc), _ptr(d_out_words), _ptr(d_out_dims), _ptr(d_status),
                                      _stream(stream))
    return _check(rc, "fdy_materialize_static") if check else rc


def tune_get(knob):
    return lib().fdy__tune_get(knob)


def tune_set(knob, value):
    return lib().fdy__tune_set(knob, value)


PROF_SLOTS = 11


PROF_SCAN_MAIN, PROF_MAT_MAIN, PROF_SCAN_OUT, PROF_SCAN_REBASE = 0, 7, 8, 9


def prof_enable(n_records, slots=None):
    """Bracket kernel launches of the library with HIP events on the caller's stream (bench
    support; 0 switches it off).  `slots`: iterable of slot numbers to record, default all."""
    mask = 0xFFFFFFFF if slots is None else sum(1 << s for s in slots)
    lib().fdy__prof_mask(mask)
    return lib().fdy__prof_enable(int(n_records))


def prof_read():
    """-> {kernel name: dict(n, total_ms, avg_ms, min_ms, max_ms)} and resets the records."""
    out = {}
    for slot in range(PROF_SLOTS):
        n, tot, mn, mx = C.c_int(0), C.c_float(0), C.c_float(0), C.c_float(0)
        if lib().fdy__prof_read(slot, C.byref(n), C.byref(tot), C.byref(mn), C.byref(mx)) != 0:
            raise FdyError(FDY_ERR_HIP, "fdy__prof_read")
        if n.value:
            out[lib().fdy__prof_name(slot).decode()] = dict(
                n=n.value, total_ms=tot.value, avg_ms=tot.value / n.value, min_ms=mn.value,
                max_ms=mx.value)
    return out


# ---- marshalling helpers -------------------------------------------------------------------
def to_device(arr, device="cuda:0"):
    """numpy array (any dtype, incl. record dtypes) -> 1-D torch.uint8 tensor on the device,
    256-byte aligned by the torch allocator."""
    import torch

    a = np.ascontiguousarray(arr)
    raw = a.reshape(-1).view(np.uint8) if a.size else np.zeros(0, np.uint8)
    return torch.from_numpy(raw.copy()).to(device)


def to_host(t, dtype, count=None):
    """torch.uint8 device tensor -> numpy array of `dtype` (first `count` records)."""
    dt = np.dtype(dtype)
    n = t.numel() // dt.itemsize if count is None else int(count)
    return t[: n * dt.itemsize].cpu().numpy().view(dt).copy()


def device_bytes(nbytes, device="cuda:0", fill=None):
    import torch

    t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device=device)
    if fill is not None:
        t.fill_(fill)
    return t


def make_mat_desc(dev, *, n_src_graphs, n_templates, n_graphs, n_maps, n_alloc, n_ranks,
                  out_words_per_map, out_nodes_total):
    """dev: dict name -> device tensor (or None) for the pointer fields of fdy_mat_desc."""
    d = fdy_mat_desc()
    d.n_src_graphs, d.n_templates, d.n_graphs = n_src_graphs, n_templates, n_graphs
    d.n_maps, d.n_alloc, d.n_ranks = n_maps, n_alloc, n_ranks
    d.out_words_per_map, d.out_nodes_total = out_words_per_map, out_nodes_total
    for name, _ in fdy_mat_desc._fields_[8:]:
        setattr(d, name, _ptr(dev.get(name)))
    return d
