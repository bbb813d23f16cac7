"""Convenience layer over the binding for tests, the smoke check and the bench (test support,
not part of the product package): uploads host arrays, allocates outputs / workspaces with
torch, calls the C-ABI entry points and brings results back.  Marshalling only - no step of
the method is computed here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2604_06664_amd as fdy

RELOC = np.dtype([("word", "<u4"), ("region", "<u4"), ("offset", "<u8")])
DEV = "cuda:0"


def _status_tensor():
    return torch.zeros(1, dtype=torch.int32, device=DEV)


def _scan_ws_bytes(n_words, n_alloc, staging=True):
    """Workspace of a scan: hierarchy and state, plus (staging) the optional staging area."""
    return fdy.fdy_scan_workspace_bytes(n_words, n_alloc) + (fdy.fdy_scan_staging_bytes(n_words) if staging else 0)


class ScanRun:
    """Device-resident inputs, outputs and workspace of one fdy_scan_pointers problem."""

    def __init__(self, words, table, capacity=None, prepared=False, staging=True):
        self.n_words = int(len(words))
        self.n_alloc = int(len(table))
        self.capacity = self.n_words if capacity is None else int(capacity)
        self.d_words = words if torch.is_tensor(words) else fdy.to_device(words)
        self.d_table = table if torch.is_tensor(table) else fdy.to_device(table)
        self.d_relocs = fdy.device_bytes(self.capacity * 16)
        self.d_count = torch.zeros(1, dtype=torch.int64, device=DEV)
        self.ws_bytes = _scan_ws_bytes(self.n_words, self.n_alloc, staging)
        self.d_ws = fdy.device_bytes(self.ws_bytes)
        self.d_status = _status_tensor()
        self.d_prepared = None
        if prepared:
            self.prepare(self.n_words)

    def prepare(self, max_words):
        """Builds the table's prepared form (fdy_scan_table_prepare); later launches pass it."""
        self.prepared_bytes = fdy.fdy_scan_table_bytes(self.n_alloc, max_words)
        self.d_prepared = fdy.device_bytes(self.prepared_bytes, fill=0xA7)
        fdy.fdy_scan_table_prepare(self.d_table, self.n_alloc, max_words, self.d_prepared,
                                   self.prepared_bytes)

    def launch(self, stream=None):
        return fdy.fdy_scan_pointers(self.d_words, self.n_words, self.d_table, self.n_alloc,
                                     self.d_relocs, self.capacity, self.d_count, self.d_prepared,
                                     self.d_ws, self.ws_bytes, self.d_status, stream)

    def result(self):
        torch.cuda.synchronize()
        count = int(self.d_count.item())
        status = int(self.d_status.item())
        relocs = fdy.to_host(self.d_relocs, RELOC, min(count, self.capacity))
        return relocs, count, status


def scan(words, table, capacity=None, prepared=False, staging=True):
    run = ScanRun(words, table, capacity, prepared=prepared, staging=staging)
    run.launch()
    return run.result()


class ScanStride4Run(ScanRun):
    """fdy_scan_pointers_stride4: `units` is a uint32 array; capacity defaults to one entry per
    position."""

    def __init__(self, units, table, capacity=None, prepared=False, staging=True):
        units = np.ascontiguousarray(units, np.uint32)
        self.n_units = int(len(units))
        self.n_alloc = int(len(table))
        self.capacity = max(self.n_units - 1, 0) if capacity is None else int(capacity)
        self.d_words = fdy.to_device(units)
        self.d_table = table if torch.is_tensor(table) else fdy.to_device(table)
        self.d_relocs = fdy.device_bytes(self.capacity * 16)
        self.d_count = torch.zeros(1, dtype=torch.int64, device=DEV)
        self.ws_bytes = _scan_ws_bytes(self.n_units, self.n_alloc, staging)
        self.d_ws = fdy.device_bytes(self.ws_bytes)
        self.d_status = _status_tensor()
        self.d_prepared = None
        if prepared:
            self.prepare(self.n_units)

    def launch(self, stream=None):
        return fdy.fdy_scan_pointers_stride4(self.d_words, self.n_units, self.d_table, self.n_alloc,
                                             self.d_relocs, self.capacity, self.d_count, self.d_prepared,
                                             self.d_ws, self.ws_bytes, self.d_status, stream)


def scan_stride4(units, table, capacity=None, prepared=False, staging=True):
    run = ScanStride4Run(units, table, capacity, prepared=prepared, staging=staging)
    run.launch()
    return run.result()


class ScanRebaseRun:
    """Device-resident inputs, output and workspace of one fdy_scan_rebase problem."""

    def __init__(self, words, table, new_base, in_place=False, n_words=None, n_alloc=None, prepared=False):
        # n_words / n_alloc: record counts when words / table are device byte tensors
        self.n_words = int(len(words) if n_words is None else n_words)
        self.n_alloc = int(len(table) if n_alloc is None else n_alloc)
        self.d_words = words if torch.is_tensor(words) else fdy.to_device(words)
        self.d_table = table if torch.is_tensor(table) else fdy.to_device(table)
        self.d_new_base = new_base if torch.is_tensor(new_base) else fdy.to_device(
            np.ascontiguousarray(new_base, np.uint64))
        self.d_out = self.d_words if in_place else fdy.device_bytes(self.n_words * 8, fill=0xEE)
        self.d_count = torch.full((1,), -1, dtype=torch.int64, device=DEV)
        self.ws_bytes = _scan_ws_bytes(self.n_words, self.n_alloc, True)
        self.d_ws = fdy.device_bytes(self.ws_bytes)
        self.d_status = _status_tensor()
        self.d_prepared = None
        if prepared:
            ScanRun.prepare(self, self.n_words)

    def launch(self, stream=None):
        return fdy.fdy_scan_rebase(self.d_words, self.n_words, self.d_table, self.n_alloc,
                                   self.d_new_base, self.d_out, self.d_count, self.d_prepared, self.d_ws,
                                   self.ws_bytes, self.d_status, stream)

    def result(self):
        torch.cuda.synchronize()
        return (fdy.to_host(self.d_out, np.uint64, self.n_words), int(self.d_count.item()),
                int(self.d_status.item()))


class ScanPointersRebaseRun(ScanRun):
    """fdy_scan_pointers_rebase: the relocation table and the rebased copy of the words."""

    def __init__(self, words, table, new_base, capacity=None, prepared=False, staging=True):
        super().__init__(words, table, capacity, prepared=prepared, staging=staging)
        self.d_new_base = new_base if torch.is_tensor(new_base) else fdy.to_device(
            np.ascontiguousarray(new_base, np.uint64))
        self.d_out = fdy.device_bytes(self.n_words * 8, fill=0xEE)

    def launch(self, stream=None):
        return fdy.fdy_scan_pointers_rebase(self.d_words, self.n_words, self.d_table, self.n_alloc,
                                            self.d_relocs, self.capacity, self.d_count, self.d_new_base,
                                            self.d_out, self.d_prepared, self.d_ws, self.ws_bytes,
                                            self.d_status, stream)

    def result(self):
        relocs, count, status = super().result()
        return relocs, count, status, fdy.to_host(self.d_out, np.uint64, self.n_words)


def scan_pointers_rebase(words, table, new_base, capacity=None, prepared=False, staging=True):
    run = ScanPointersRebaseRun(words, table, new_base, capacity, prepared=prepared, staging=staging)
    run.launch()
    return run.result()


def scan_rebase(words, table, new_base, in_place=False, prepared=False):
    run = ScanRebaseRun(words, table, new_base, in_place, prepared=prepared)
    run.launch()
    return run.result()


def reloc_segment(d_relocs, d_count, capacity, word_off):
    d_off = fdy.to_device(np.ascontiguousarray(word_off, np.uint64))
    d_out = fdy.device_bytes(len(word_off) * 8, fill=0xEE)
    fdy.fdy_reloc_segment(d_relocs, d_count, capacity, d_off, len(word_off), d_out)
    torch.cuda.synchronize()
    return fdy.to_host(d_out, np.uint64, len(word_off)), d_out


def fingerprint(nodes, node_off, mask, want_tmpl_graph=True):
    G = len(node_off) - 1
    d_nodes = fdy.to_device(nodes)
    d_off = fdy.to_device(np.ascontiguousarray(node_off, np.uint64))
    d_keys = fdy.device_bytes(G * 8, fill=0xEE)
    d_tid = fdy.device_bytes(G * 4, fill=0xEE)
    d_tg = fdy.device_bytes(G * 4, fill=0xEE) if want_tmpl_graph else None
    d_nt = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    ws_bytes = fdy.fdy_fingerprint_workspace_bytes(G)
    d_ws = fdy.device_bytes(ws_bytes, fill=0x3C)
    fdy.fdy_fingerprint(d_nodes, d_off, G, mask, d_keys, d_tid, d_tg, d_nt, d_workspace=d_ws,
                        workspace_bytes=ws_bytes)
    torch.cuda.synchronize()
    nt = int(d_nt.item())
    keys = fdy.to_host(d_keys, np.uint64, G)
    tid = fdy.to_host(d_tid, np.uint32, G)
    tg = fdy.to_host(d_tg, np.uint32, nt) if want_tmpl_graph else None
    return keys, tid, tg, dict(d_keys=d_keys, d_tid=d_tid, d_tg=d_tg, d_nt=d_nt)


def derive_overrides(words, word_off, graph_tmpl, tmpl_graph, capacity=None):
    """-> (ovr OVR32[min(total, capacity)], ovr_off u64[G+1], status)"""
    from synth import layout as L

    words = np.ascontiguousarray(words, np.uint64)
    word_off = np.ascontiguousarray(word_off, np.uint64)
    gt = np.ascontiguousarray(graph_tmpl, np.uint32)
    tg = np.ascontiguousarray(tmpl_graph, np.uint32)
    G, W = len(gt), len(words)
    cap = 2 * W if capacity is None else int(capacity)
    d_words, d_off = fdy.to_device(words), fdy.to_device(word_off)
    d_gt, d_tg = fdy.to_device(gt), fdy.to_device(tg)
    d_ovr = fdy.device_bytes(cap * 8, fill=0xEE)
    d_ovr_off = fdy.device_bytes((G + 1) * 8, fill=0xEE)
    ws_bytes = fdy.fdy_derive_workspace_bytes(W, G)
    d_ws = fdy.device_bytes(ws_bytes)
    d_status = _status_tensor()
    fdy.fdy_derive_overrides(d_words, W, d_off, G, d_gt, d_tg, len(tg), d_ovr, cap, d_ovr_off, d_ws,
                             ws_bytes, d_status)
    torch.cuda.synchronize()
    off = fdy.to_host(d_ovr_off, np.uint64, G + 1)
    return fdy.to_host(d_ovr, L.OVR32, min(int(off[G]), cap)), off, int(d_status.item())


class MatRun:
    """Device-resident inputs, outputs and workspace of one fdy_materialize problem.
    `mp` is a synth.MatProblem (host arrays); `device_overrides` may replace uploaded arrays
    by tensors that are already on the device (e.g. relocs straight from a scan)."""

    def __init__(self, mp, want_dims=True, device_overrides=None, poison=True, out=None):
        self.mp = mp
        dev = dict(device_overrides or {})
        for name in mp.ARRAYS:
            if name not in dev:
                v = getattr(mp, name)
                dev[name] = None if v is None else fdy.to_device(v)
        self.dev = dev
        self.wpm = mp.out_words_per_map()
        self.nodes_total = mp.out_nodes_total() if want_dims else 0
        self.desc = fdy.make_mat_desc(
            dev, n_src_graphs=mp.S, n_templates=mp.T, n_graphs=mp.G, n_maps=mp.M, n_alloc=mp.A,
            n_ranks=mp.n_ranks, out_words_per_map=self.wpm, out_nodes_total=self.nodes_total)
        self.d_out = out if out is not None else fdy.device_bytes(mp.M * self.wpm * 8,
                                                                  fill=0xCD if poison else None)
        self.d_dims = (fdy.device_bytes(self.nodes_total * 24, fill=0xCD if poison else None)
                       if want_dims else None)
        self.ws_bytes = fdy.fdy_materialize_workspace_bytes(self.desc)
        self.d_ws = fdy.device_bytes(self.ws_bytes)
        self.d_status = _status_tensor()

    def launch(self, stream=None, check=True):
        return fdy.fdy_materialize(self.desc, self.d_out, self.d_dims, self.d_ws, self.ws_bytes,
                                   self.d_status, stream, check=check)

    def result(self):
        torch.cuda.synchronize()
        out = fdy.to_host(self.d_out, np.uint64, self.mp.M * self.wpm).reshape(self.mp.M, self.wpm)
        dims = (fdy.to_host(self.d_dims, np.uint32, self.nodes_total * 6).reshape(-1, 6)
                if self.d_dims is not None else None)
        return out, dims, int(self.d_status.item())


def materialize(mp, want_dims=True):
    """One materialization, run both ways the library has for it (tiles resolved by a launch of
    their own / by the main kernel's workgroups, which small launches choose by themselves): the
    two must agree in every byte and in the status word; the result is returned once."""
    res = []
    for self_wgs in (0, None):
        old = fdy.tune_set(fdy.TUNE_MAT_SELF_WGS, self_wgs) if self_wgs is not None else None
        try:
            run = MatRun(mp, want_dims)
            run.launch()
            res.append(run.result())
        finally:
            if old is not None:
                fdy.tune_set(fdy.TUNE_MAT_SELF_WGS, old)
    (out0, dims0, st0), (out1, dims1, st1) = res
    from synth import layout as L

    if (st0 | st1) & L.ST_BAD_ORDER:
        # a list out of order: both say so; which entries then count as misplaced, and what is
        # written, depends on how the slices were searched and is unspecified
        assert (st0 & ~L.ST_BAD_INDEX) == (st1 & ~L.ST_BAD_INDEX), (st0, st1)
        return res[1]
    assert st0 == st1, (st0, st1)
    assert np.array_equal(out0, out1)
    if want_dims:
        assert np.array_equal(dims0, dims1)
    return res[1]


class PathRun:
    """The whole hot path for one capture archive, device-resident and chained on one stream
    without host round trips: scan -> reloc segmentation -> fingerprint -> materialize.
    `ar` is a synth.Archive; `reloc_capacity` bounds the relocation table (host knowledge:
    at most one entry per word)."""

    def __init__(self, ar, reloc_capacity=None, want_dims=True, maps=None, one_pass=None, prepared=True):
        """one_pass: the scan itself writes the materialized output (fdy_scan_pointers_rebase) and
        fdy_materialize is not called.  That is the whole of (c) when every graph is its own
        template and there is one base map and nothing to override or patch; None = use it
        exactly then.  prepared: the allocation table's search hierarchy is built once, here
        (fdy_scan_table_prepare), not by every step; relocation segmentation and fingerprint
        are then one launch (fdy_segment_fingerprint)."""
        from synth import MatProblem

        self.ar = ar
        G = ar.n_graphs
        self.G = G
        cap = len(ar.words) if reloc_capacity is None else int(reloc_capacity)
        own = (ar.n_templates == G and np.array_equal(ar.graph_tmpl, np.arange(G))
               and np.array_equal(ar.tmpl_graph, np.arange(G)))
        can = bool(own and ar.n_maps == 1 and maps is None and len(ar.ovr) == 0 and len(ar.govr) == 0
                   and len(ar.patch) == 0 and len(ar.nodes) == 0)
        self.one_pass = can if one_pass is None else bool(one_pass)
        assert can or not self.one_pass
        self.prepared = bool(prepared)
        if self.one_pass:
            self.scan = ScanPointersRebaseRun(ar.words, ar.table, ar.new_base[0], cap, prepared=prepared)
        else:
            self.scan = ScanRun(ar.words, ar.table, cap, prepared=prepared)
        self.d_word_off = fdy.to_device(ar.word_off)
        self.d_reloc_off = fdy.device_bytes((G + 1) * 8, fill=0xEE)
        self.d_nodes = fdy.to_device(ar.nodes)
        self.d_node_off = fdy.to_device(ar.node_off)
        self.d_keys = fdy.device_bytes(G * 8, fill=0xEE)
        self.d_tid = fdy.device_bytes(G * 4, fill=0xEE)
        self.d_tg = fdy.device_bytes(G * 4, fill=0xEE)
        self.d_nt = torch.full((1,), -1, dtype=torch.int32, device=DEV)
        # host-side manifest knowledge (template of each graph) sizes the output; the device
        # arrays the kernels consume are the ones fdy_fingerprint writes
        empty_rel = np.zeros(0, RELOC)
        mp = MatProblem.from_archive(ar, empty_rel, np.zeros(G + 1, np.uint64), maps=maps)
        self.mat = MatRun(mp, want_dims=want_dims and len(ar.nodes) > 0, device_overrides=dict(
            src_words=self.scan.d_words, relocs=self.scan.d_relocs, src_reloc_off=self.d_reloc_off,
            src_nodes=self.d_nodes, src_node_off=self.d_node_off, graph_tmpl=self.d_tid,
            tmpl_graph=self.d_tg), out=self.scan.d_out if self.one_pass else None)

    def step(self, stream=None):
        ar = self.ar
        self.scan.launch(stream)
        if self.prepared:
            fdy.fdy_segment_fingerprint(self.scan.d_relocs, self.scan.d_count, self.scan.capacity,
                                        self.d_word_off, self.d_reloc_off, self.d_nodes, self.d_node_off,
                                        self.G, ar.fp_mask, self.d_keys, self.d_tid, self.d_tg, self.d_nt,
                                        d_prepared=self.scan.d_prepared, stream=stream)
        else:
            fdy.fdy_reloc_segment(self.scan.d_relocs, self.scan.d_count, self.scan.capacity,
                                  self.d_word_off, self.G + 1, self.d_reloc_off, stream)
            fdy.fdy_fingerprint(self.d_nodes, self.d_node_off, self.G, ar.fp_mask, self.d_keys,
                                self.d_tid, self.d_tg, self.d_nt, stream)
        if not self.one_pass:
            self.mat.launch(stream)

    def status(self):
        torch.cuda.synchronize()
        return int(self.scan.d_status.item()) | int(self.mat.d_status.item())
