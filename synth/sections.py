"""Section lists of the binary archive form, assembled from a synthetic archive.

Data wrangling only (selecting and concatenating arrays, shifting word indices when graphs
are dropped); none of the method's arithmetic.  The kind numbers are those of
include/fdy_archive.h.
"""
from __future__ import annotations

import numpy as np

from . import layout as L

(SEC_TABLE, SEC_WORDS, SEC_WORD_OFF, SEC_NODES, SEC_NODE_OFF, SEC_RELOCS, SEC_RELOC_OFF, SEC_GRAPH_TMPL,
 SEC_TMPL_GRAPH, SEC_OVR, SEC_OVR_OFF, SEC_GOVR, SEC_GOVR_OFF, SEC_PATCH, SEC_PATCH_OFF, SEC_KEYS) = range(1, 17)

U64 = np.uint64


def archive_sections(ar, relocs, reloc_off, keys=None, compact=False):
    """[(kind, array)] for archive `ar` whose words were scanned into `relocs`, segmented per
    graph by `reloc_off`.  compact: store only the template graphs (S = T); otherwise every
    captured graph is stored (S = G)."""
    word_off = ar.word_off.astype(np.int64)
    node_off = ar.node_off.astype(np.int64)
    reloc_off = np.asarray(reloc_off).astype(np.int64)
    tmpl_graph = ar.tmpl_graph.astype(np.uint32)
    words, nodes, relocs = ar.words, ar.nodes, np.asarray(relocs, L.RELOC)
    if compact:
        keep = ar.tmpl_graph.astype(np.int64)
        nw = word_off[keep + 1] - word_off[keep]
        new_word_off = np.concatenate([[0], np.cumsum(nw)])
        words = np.concatenate([ar.words[word_off[s]:word_off[s + 1]] for s in keep])
        nodes = np.concatenate([ar.nodes[node_off[s]:node_off[s + 1]] for s in keep])
        parts = []
        for i, s in enumerate(keep):
            r = relocs[reloc_off[s]:reloc_off[s + 1]].copy()
            r["word"] = (r["word"].astype(np.int64) - word_off[s] + new_word_off[i]).astype(np.uint32)
            parts.append(r)
        relocs = np.concatenate(parts)
        reloc_off = np.concatenate([[0], np.cumsum([len(p) for p in parts])])
        node_off = np.concatenate([[0], np.cumsum(node_off[keep + 1] - node_off[keep])])
        word_off = new_word_off
        tmpl_graph = np.arange(len(keep), dtype=np.uint32)
    secs = [
        (SEC_TABLE, ar.table),
        (SEC_WORDS, words.astype(U64)),
        (SEC_WORD_OFF, word_off.astype(U64)),
        (SEC_NODES, nodes),
        (SEC_NODE_OFF, node_off.astype(U64)),
        (SEC_RELOCS, relocs),
        (SEC_RELOC_OFF, reloc_off.astype(U64)),
        (SEC_GRAPH_TMPL, ar.graph_tmpl.astype(np.uint32)),
        (SEC_TMPL_GRAPH, tmpl_graph),
        (SEC_OVR, ar.ovr),
        (SEC_OVR_OFF, ar.ovr_off.astype(U64)),
        (SEC_GOVR, ar.govr),
        (SEC_GOVR_OFF, ar.govr_off.astype(U64)),
    ]
    if ar.n_ranks:
        secs += [(SEC_PATCH, ar.patch), (SEC_PATCH_OFF, ar.patch_off.astype(U64))]
    if keys is not None:
        secs.append((SEC_KEYS, np.asarray(keys, U64)))
    return secs
