"""Oracle of the binary archive format (the layout stated in include/fdy_archive.h).

TEST INFRASTRUCTURE ONLY, like the rest of this package.  Plain numpy / struct code written
from the format's description, independent of the library's reader and writer:

  checksum(data)            the position-weighted word sum
  build(sections)           -> the bytes of an archive file
  parse(blob, verify)       -> {kind: raw bytes of the section}; raises FormatError / ChecksumError
  check(sections)           -> info dict; raises ContentError with the broken rule

The paper (Section 5.3, last paragraph; Section 6.5) states only that a binary form exists
and that 512 graphs parse in under 100 ms; the layout is this repository's own, so the pins
of this module are hand-worked byte values and closed forms of the checksum (tests).
"""
from __future__ import annotations

import struct

import numpy as np

from synth import layout as L

MAGIC = b"FDYARCH1"
VERSION = 1
MAX_SECTIONS = 64
HEADER_BYTES, DIR_BYTES, BODY_ALIGN, SECTION_ALIGN = 64, 32, 4096, 256

(TABLE, WORDS, WORD_OFF, NODES, NODE_OFF, RELOCS, RELOC_OFF, GRAPH_TMPL, TMPL_GRAPH, OVR, OVR_OFF, GOVR,
 GOVR_OFF, PATCH, PATCH_OFF, KEYS) = range(1, 17)

DTYPES = {
    TABLE: L.ALLOC, WORDS: np.dtype("<u8"), WORD_OFF: np.dtype("<u8"), NODES: L.NODE, NODE_OFF: np.dtype("<u8"),
    RELOCS: L.RELOC, RELOC_OFF: np.dtype("<u8"), GRAPH_TMPL: np.dtype("<u4"), TMPL_GRAPH: np.dtype("<u4"),
    OVR: L.OVR32, OVR_OFF: np.dtype("<u8"), GOVR: L.GRID_OVR, GOVR_OFF: np.dtype("<u8"), PATCH: L.PATCH,
    PATCH_OFF: np.dtype("<u8"), KEYS: np.dtype("<u8"),
}


class FormatError(ValueError):
    pass


class ChecksumError(ValueError):
    pass


class ContentError(ValueError):
    pass


def _pad(n, a):
    return -(-n // a) * a


def checksum(data):
    """Bytes zero-padded to whole 64-bit little-endian words w[i]: sum of w[i] * (2 i + 1) mod 2^64."""
    raw = bytes(data)
    raw += b"\0" * (-len(raw) % 8)
    w = np.frombuffer(raw, "<u8")
    k = np.arange(len(w), dtype=np.uint64) * np.uint64(2) + np.uint64(1)
    with np.errstate(over="ignore"):
        return int((w * k).sum(dtype=np.uint64))


def build(sections):
    """sections: list of (kind, numpy array of the kind's record type).  -> bytes of the file."""
    n = len(sections)
    assert n <= MAX_SECTIONS
    body_offset = _pad(HEADER_BYTES + DIR_BYTES * n, BODY_ALIGN)
    directory, payloads, cursor = b"", [], body_offset
    for kind, arr in sections:
        a = np.ascontiguousarray(arr)
        assert a.dtype.itemsize == DTYPES[kind].itemsize
        raw = a.tobytes()
        directory += struct.pack("<IIQQQ", kind, a.dtype.itemsize, cursor, a.size, checksum(raw))
        payloads.append(raw + b"\0" * (_pad(len(raw), SECTION_ALIGN) - len(raw)))
        cursor += _pad(len(raw), SECTION_ALIGN)

    def header(head_sum):
        return MAGIC + struct.pack("<IIQQQQQQ", VERSION, n, cursor, body_offset, cursor - body_offset, head_sum, 0, 0)

    head = header(checksum(header(0) + directory)) + directory
    return head + b"\0" * (body_offset - len(head)) + b"".join(payloads)


def parse(blob, verify=True):
    """-> dict kind -> numpy record array (a copy).  Applies every container rule."""
    if len(blob) < HEADER_BYTES:
        raise FormatError("shorter than a header")
    if blob[:8] != MAGIC:
        raise FormatError("magic")
    version, n, file_bytes, body_offset, body_bytes, head_sum, r0, r1 = struct.unpack_from("<IIQQQQQQ", blob, 8)
    if version != VERSION:
        raise FormatError("version")
    if file_bytes != len(blob):
        raise FormatError("file size")
    if n > MAX_SECTIONS or HEADER_BYTES + DIR_BYTES * n > len(blob):
        raise FormatError("section count")
    if body_offset % BODY_ALIGN or body_offset < HEADER_BYTES + DIR_BYTES * n or body_offset > file_bytes:
        raise FormatError("body offset")
    if body_bytes != file_bytes - body_offset:
        raise FormatError("body size")
    if r0 or r1:
        raise FormatError("reserved")
    entries = [struct.unpack_from("<IIQQQ", blob, HEADER_BYTES + DIR_BYTES * i) for i in range(n)]
    cursor, seen = body_offset, set()
    for kind, eb, off, count, _ in entries:
        if kind not in DTYPES:
            raise FormatError("unknown kind")
        if kind in seen:
            raise FormatError("kind twice")
        seen.add(kind)
        if eb != DTYPES[kind].itemsize:
            raise FormatError("element size")
        if off % SECTION_ALIGN or off < cursor:
            raise FormatError("offset")
        if off > file_bytes or _pad(count * eb, SECTION_ALIGN) > file_bytes - off:
            raise FormatError("past the end")
        cursor = off + _pad(count * eb, SECTION_ALIGN)
    if cursor != file_bytes:
        raise FormatError("trailing bytes")
    zeroed = bytearray(blob[: HEADER_BYTES + DIR_BYTES * n])
    zeroed[40:48] = b"\0" * 8
    if checksum(zeroed) != head_sum:
        raise ChecksumError("header")
    out = {}
    for kind, eb, off, count, s in entries:
        raw = blob[off: off + count * eb]
        if verify and checksum(raw) != s:
            raise ChecksumError(f"section {kind}")
        out[kind] = np.frombuffer(raw, DTYPES[kind]).copy()
    return out


def _offsets(name, off, length, total):
    if len(off) != length:
        raise ContentError(f"{name}: length")
    if off[0] != 0:
        raise ContentError(f"{name}: start")
    if np.any(off[1:] < off[:-1]):
        raise ContentError(f"{name}: decreases")
    if off[-1] != total:
        raise ContentError(f"{name}: end")


def _ascending_per_slice(name, loc, off):
    """loc strictly ascending inside each slice [off[i], off[i+1])."""
    if len(loc) < 2:
        return
    not_asc = np.flatnonzero(loc[1:] <= loc[:-1]) + 1  # positions whose predecessor is not smaller
    starts = set(int(x) for x in off)
    for i in not_asc:
        if int(i) not in starts:
            raise ContentError(f"{name}: not ascending at {int(i)}")


def check(sec):
    """sec: dict kind -> record array.  The content rules, one after another.  -> info dict."""
    for k in (TABLE, WORDS, WORD_OFF, NODES, NODE_OFF, RELOCS, RELOC_OFF, GRAPH_TMPL, TMPL_GRAPH, OVR, OVR_OFF,
              GOVR, GOVR_OFF):
        if k not in sec:
            raise ContentError("missing section")
    if (PATCH in sec) != (PATCH_OFF in sec):
        raise ContentError("patch pair")
    table, words, word_off = sec[TABLE], sec[WORDS], sec[WORD_OFF].astype(np.int64)
    nodes, node_off = sec[NODES], sec[NODE_OFF].astype(np.int64)
    relocs, reloc_off = sec[RELOCS], sec[RELOC_OFF].astype(np.int64)
    graph_tmpl, tmpl_graph = sec[GRAPH_TMPL].astype(np.int64), sec[TMPL_GRAPH].astype(np.int64)
    A, S, T, G = len(table), len(word_off) - 1, len(tmpl_graph), len(graph_tmpl)
    limit = 1 << 20
    if A < 1 or A >= 1 << 32:
        raise ContentError("table count")
    base = [int(x) for x in table["base"]]
    size = [int(x) for x in table["size"]]
    for i in range(A):
        if size[i] < 1 or base[i] + size[i] >= 1 << 64:  # the end must be a representable address
            raise ContentError("table entry size / wrap")
        if i and base[i] < base[i - 1] + size[i - 1]:
            raise ContentError("table order / overlap")
    if S < 1 or S > limit or T < 1 or T > limit or G < 1 or G > limit:
        raise ContentError("graph counts")
    if len(words) >= 1 << 32:
        raise ContentError("too many words")
    _offsets("WORD_OFF", word_off, S + 1, len(words))
    _offsets("NODE_OFF", node_off, S + 1, len(nodes))
    _offsets("RELOC_OFF", reloc_off, S + 1, len(relocs))
    blob_len = nodes["blob_len"].astype(np.int64)
    if np.any(blob_len % 8):
        raise ContentError("blob length not a multiple of 8")
    csum = np.concatenate([[0], np.cumsum(blob_len)])
    if np.any(csum[node_off[1:]] - csum[node_off[:-1]] != 8 * (word_off[1:] - word_off[:-1])):
        raise ContentError("blob lengths do not add up")
    rw = relocs["word"].astype(np.int64)
    graph_of_reloc = np.repeat(np.arange(S), reloc_off[1:] - reloc_off[:-1])
    if np.any(rw < word_off[graph_of_reloc]) or np.any(rw >= word_off[graph_of_reloc + 1]):
        raise ContentError("reloc outside its graph")
    _ascending_per_slice("RELOCS", rw, reloc_off)
    region = relocs["region"].astype(np.int64)
    if np.any(region >= A):
        raise ContentError("reloc region")
    if np.any(relocs["offset"] >= table["size"][region]):
        raise ContentError("reloc offset")
    with np.errstate(over="ignore"):
        if np.any(words[rw] != table["base"][region] + relocs["offset"]):
            raise ContentError("reloc does not match its word")
    if np.any(tmpl_graph >= S):
        raise ContentError("tmpl_graph")
    if np.any(graph_tmpl >= T):
        raise ContentError("graph_tmpl")
    src = tmpl_graph[graph_tmpl]
    g_words = word_off[src + 1] - word_off[src]
    g_nodes = node_off[src + 1] - node_off[src]

    ovr, ovr_off = sec[OVR], sec[OVR_OFF].astype(np.int64)
    _offsets("OVR_OFF", ovr_off, G + 1, len(ovr))
    g_of = np.repeat(np.arange(G), ovr_off[1:] - ovr_off[:-1])
    bo = ovr["byte_off"].astype(np.int64)
    if np.any(bo % 4) or np.any(bo >= 8 * g_words[g_of]):
        raise ContentError("override misaligned or outside the blob")
    _ascending_per_slice("OVR", bo, ovr_off)

    govr, govr_off = sec[GOVR], sec[GOVR_OFF].astype(np.int64)
    _offsets("GOVR_OFF", govr_off, G + 1, len(govr))
    g_of = np.repeat(np.arange(G), govr_off[1:] - govr_off[:-1])
    gn = govr["node"].astype(np.int64)
    if np.any(gn >= g_nodes[g_of]):
        raise ContentError("grid override outside the nodes")
    _ascending_per_slice("GOVR", gn, govr_off)

    R = 0
    if PATCH in sec:
        patch, patch_off = sec[PATCH], sec[PATCH_OFF].astype(np.int64)
        if len(patch_off) < 2 or (len(patch_off) - 1) % T:
            raise ContentError("PATCH_OFF: length")
        R = (len(patch_off) - 1) // T
        if R > 0xFFFF:
            raise ContentError("rank count")
        _offsets("PATCH_OFF", patch_off, T * R + 1, len(patch))
        t_of = np.repeat(np.arange(T * R) // R, patch_off[1:] - patch_off[:-1])
        t_words = word_off[tmpl_graph + 1] - word_off[tmpl_graph]
        pw = patch["word"].astype(np.int64)
        if np.any(pw >= t_words[t_of]) or np.any(patch["reserved"] != 0):
            raise ContentError("patch outside the template or reserved set")
        _ascending_per_slice("PATCH", pw, patch_off)
    if KEYS in sec:
        keys = sec[KEYS]
        if len(keys) != G:
            raise ContentError("KEYS: length")
        key_to_t, t_to_key = {}, {}
        for k, t in zip(keys.tolist(), graph_tmpl.tolist()):
            if key_to_t.setdefault(k, t) != t or t_to_key.setdefault(t, k) != k:
                raise ContentError("KEYS: keys and templates disagree")
    return dict(n_src_graphs=S, n_templates=T, n_graphs=G, n_ranks=R, n_alloc=A, n_words=len(words),
                n_nodes=len(nodes), n_relocs=len(relocs), out_words_per_map=int(g_words.sum()),
                out_nodes_total=int(g_nodes.sum()))
