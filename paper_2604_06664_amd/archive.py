"""Binding of include/fdy_archive.h (the binary on-disk archive): same names, marshalling only."""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import FDY_ERR_HIP, FDY_ERR_INVALID_ARG, FDY_OK, FdyError, _ptr, _stream, fdy_mat_desc, lib  # noqa: F401

FDY_ERR_IO, FDY_ERR_FORMAT, FDY_ERR_CHECKSUM, FDY_ERR_CONTENT = -7, -8, -9, -10
FDY_ARCHIVE_VERIFY_SUMS = 1

(FDY_SEC_TABLE, FDY_SEC_WORDS, FDY_SEC_WORD_OFF, FDY_SEC_NODES, FDY_SEC_NODE_OFF, FDY_SEC_RELOCS,
 FDY_SEC_RELOC_OFF, FDY_SEC_GRAPH_TMPL, FDY_SEC_TMPL_GRAPH, FDY_SEC_OVR, FDY_SEC_OVR_OFF, FDY_SEC_GOVR,
 FDY_SEC_GOVR_OFF, FDY_SEC_PATCH, FDY_SEC_PATCH_OFF, FDY_SEC_KEYS) = range(1, 17)


class fdy_archive_src(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("elem_bytes", C.c_uint32), ("count", C.c_uint64), ("data", C.c_void_p)]


class fdy_archive_info(C.Structure):
    _fields_ = ([(n, C.c_uint32) for n in ("n_src_graphs", "n_templates", "n_graphs", "n_ranks", "n_alloc",
                                           "reserved")]
                + [(n, C.c_uint64) for n in ("n_words", "n_nodes", "n_relocs", "out_words_per_map",
                                             "out_nodes_total")])


_declared = False


def _L():
    global _declared
    L = lib()
    if not _declared:
        L.fdy_archive_elem_bytes.restype = C.c_uint32
        L.fdy_archive_elem_bytes.argtypes = [C.c_uint32]
        L.fdy_archive_sum.restype = C.c_uint64
        L.fdy_archive_sum.argtypes = [C.c_void_p, C.c_size_t]
        L.fdy_archive_write.restype = C.c_int
        L.fdy_archive_write.argtypes = [C.c_char_p, C.POINTER(fdy_archive_src), C.c_uint32]
        L.fdy_archive_open.restype = C.c_int
        L.fdy_archive_open.argtypes = [C.c_char_p, C.c_uint32, C.POINTER(C.c_void_p)]
        L.fdy_archive_close.restype = C.c_int
        L.fdy_archive_close.argtypes = [C.c_void_p]
        L.fdy_archive_last_failure.restype = C.c_char_p
        L.fdy_archive_section_count.restype = C.c_uint32
        L.fdy_archive_section_count.argtypes = [C.c_void_p]
        L.fdy_archive_file_bytes.restype = C.c_uint64
        L.fdy_archive_file_bytes.argtypes = [C.c_void_p]
        L.fdy_archive_body_bytes.restype = C.c_uint64
        L.fdy_archive_body_bytes.argtypes = [C.c_void_p]
        L.fdy_archive_section.restype = C.c_int
        L.fdy_archive_section.argtypes = [C.c_void_p, C.c_uint32, C.POINTER(C.c_void_p), C.POINTER(C.c_uint64),
                                          C.POINTER(C.c_uint32)]
        L.fdy_archive_check.restype = C.c_int
        L.fdy_archive_check.argtypes = [C.c_void_p, C.POINTER(fdy_archive_info)]
        L.fdy_archive_upload.restype = C.c_int
        L.fdy_archive_upload.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.fdy_archive_device_section.restype = C.c_void_p
        L.fdy_archive_device_section.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p]
        L.fdy_archive_mat_desc.restype = C.c_int
        L.fdy_archive_mat_desc.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(fdy_mat_desc)]
        _declared = True
    return L


def _check(rc, where):
    if rc != FDY_OK:
        err = FdyError(rc, where)
        err.args = (f"{err.args[0]}: {fdy_archive_last_failure()}",)
        raise err
    return rc


def fdy_archive_elem_bytes(kind):
    return _L().fdy_archive_elem_bytes(int(kind))


def fdy_archive_sum(h_bytes):
    """h_bytes: bytes-like or numpy array in host memory."""
    a = np.frombuffer(h_bytes, np.uint8) if not isinstance(h_bytes, np.ndarray) else np.ascontiguousarray(h_bytes)
    return _L().fdy_archive_sum(a.ctypes.data if a.size else None, a.nbytes)


def fdy_archive_last_failure():
    return _L().fdy_archive_last_failure().decode()


def fdy_archive_write(path, sections, check=True):
    """sections: iterable of (kind, numpy array) in host memory, or (kind, elem_bytes, array) to
    pass an element size other than the array's own (error-path tests)."""
    keep, srcs = [], []
    for sec in sections:
        kind, arr = sec[0], np.ascontiguousarray(sec[-1])
        eb = sec[1] if len(sec) == 3 else arr.dtype.itemsize
        keep.append(arr)
        srcs.append(fdy_archive_src(int(kind), int(eb), arr.size, arr.ctypes.data if arr.size else None))
    arr_t = (fdy_archive_src * max(len(srcs), 1))(*srcs)
    rc = _L().fdy_archive_write(str(path).encode(), arr_t, len(srcs))
    return _check(rc, "fdy_archive_write") if check else rc


def fdy_archive_open(path, flags=0, check=True):
    """-> opaque handle (int) to pass to the other calls; (rc, None) style when check=False."""
    h = C.c_void_p(None)
    rc = _L().fdy_archive_open(str(path).encode(), int(flags), C.byref(h))
    if check:
        _check(rc, "fdy_archive_open")
        return h.value
    return rc, h.value


def fdy_archive_close(a):
    return _L().fdy_archive_close(a)


def fdy_archive_section_count(a):
    return _L().fdy_archive_section_count(a)


def fdy_archive_file_bytes(a):
    return _L().fdy_archive_file_bytes(a)


def fdy_archive_body_bytes(a):
    return _L().fdy_archive_body_bytes(a)


def fdy_archive_section(a, kind, dtype=None):
    """-> numpy array copied out of the mapping (records of `dtype`, default raw bytes), or None
    if the archive has no such section."""
    p, n, eb = C.c_void_p(None), C.c_uint64(0), C.c_uint32(0)
    if _L().fdy_archive_section(a, int(kind), C.byref(p), C.byref(n), C.byref(eb)) != FDY_OK:
        return None
    nbytes = n.value * eb.value
    raw = np.ctypeslib.as_array(C.cast(p, C.POINTER(C.c_uint8)), shape=(nbytes,)).copy() if nbytes else \
        np.zeros(0, np.uint8)
    if dtype is None:
        return raw
    dt = np.dtype(dtype)
    assert dt.itemsize == eb.value
    return raw.view(dt)


def fdy_archive_check(a, check=True):
    """-> fdy_archive_info; (rc, info) when check=False."""
    info = fdy_archive_info()
    rc = _L().fdy_archive_check(a, C.byref(info))
    if check:
        _check(rc, "fdy_archive_check")
        return info
    return rc, info


def fdy_archive_upload(a, d_slab, slab_bytes, stream=None, check=True):
    rc = _L().fdy_archive_upload(a, _ptr(d_slab), int(slab_bytes), _stream(stream))
    return _check(rc, "fdy_archive_upload") if check else rc


def fdy_archive_device_section(a, kind, d_slab):
    return _L().fdy_archive_device_section(a, int(kind), _ptr(d_slab))


def fdy_archive_mat_desc(a, d_slab, h_desc=None, check=True):
    d = fdy_mat_desc() if h_desc is None else h_desc
    rc = _L().fdy_archive_mat_desc(a, _ptr(d_slab), C.byref(d))
    if check:
        _check(rc, "fdy_archive_mat_desc")
        return d
    return rc, d
