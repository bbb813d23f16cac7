"""Host-side container of one materialize problem: the arrays `fdy_materialize` takes
(field meanings as in include/fdy.h), as contiguous numpy arrays.  Input description only;
both the oracle binding and the HIP binding marshal it, neither's arithmetic lives here."""
from __future__ import annotations

import numpy as np

from . import layout as L


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


class MatProblem:
    ARRAYS = ("src_words", "src_word_off", "src_nodes", "src_node_off", "relocs", "src_reloc_off",
              "tmpl_graph", "graph_tmpl", "ovr", "ovr_off", "govr", "govr_off", "new_base",
              "map_rank", "patch", "patch_off")

    def __init__(self, *, src_words, src_word_off, src_nodes, src_node_off, relocs, src_reloc_off,
                 tmpl_graph, graph_tmpl, ovr, ovr_off, govr, govr_off, new_base, map_rank, n_ranks,
                 patch, patch_off):
        self.src_words = _c(src_words, np.uint64)
        self.src_word_off = _c(src_word_off, np.uint64)
        self.src_nodes = _c(src_nodes, L.NODE)
        self.src_node_off = _c(src_node_off, np.uint64)
        self.relocs = _c(relocs, L.RELOC)
        self.src_reloc_off = _c(src_reloc_off, np.uint64)
        self.tmpl_graph = _c(tmpl_graph, np.uint32)
        self.graph_tmpl = _c(graph_tmpl, np.uint32)
        self.ovr = _c(ovr, L.OVR32)
        self.ovr_off = _c(ovr_off, np.uint64)
        self.govr = _c(govr, L.GRID_OVR)
        self.govr_off = _c(govr_off, np.uint64)
        self.new_base = _c(new_base, np.uint64)
        assert self.new_base.ndim == 2
        self.map_rank = None if map_rank is None else _c(map_rank, np.uint32)
        self.n_ranks = int(n_ranks) if map_rank is not None else 0
        self.patch = _c(patch, L.PATCH)
        self.patch_off = _c(patch_off, np.uint64)

    @property
    def S(self):
        return len(self.src_word_off) - 1

    @property
    def T(self):
        return len(self.tmpl_graph)

    @property
    def G(self):
        return len(self.graph_tmpl)

    @property
    def M(self):
        return self.new_base.shape[0]

    @property
    def A(self):
        return self.new_base.shape[1]

    def out_words_per_map(self):
        nw = np.diff(self.src_word_off.astype(np.int64))
        return int(nw[self.tmpl_graph[self.graph_tmpl]].sum())

    def out_nodes_total(self):
        nn = np.diff(self.src_node_off.astype(np.int64))
        return int(nn[self.tmpl_graph[self.graph_tmpl]].sum())

    @classmethod
    def from_archive(cls, ar, relocs, reloc_off, graph_tmpl=None, tmpl_graph=None, maps=None):
        """The archive as source, its graphs as outputs; relocs/reloc_off from a scan of
        ar.words and its segmentation by ar.word_off."""
        nb = ar.new_base if maps is None else ar.new_base[maps]
        mr = ar.map_rank if (maps is None or ar.map_rank is None) else ar.map_rank[maps]
        return cls(src_words=ar.words, src_word_off=ar.word_off, src_nodes=ar.nodes,
                   src_node_off=ar.node_off, relocs=relocs, src_reloc_off=reloc_off,
                   tmpl_graph=ar.tmpl_graph if tmpl_graph is None else tmpl_graph,
                   graph_tmpl=ar.graph_tmpl if graph_tmpl is None else graph_tmpl,
                   ovr=ar.ovr, ovr_off=ar.ovr_off, govr=ar.govr, govr_off=ar.govr_off,
                   new_base=nb, map_rank=mr, n_ranks=ar.n_ranks, patch=ar.patch,
                   patch_off=ar.patch_off)
