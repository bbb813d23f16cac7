"""Pins for the oracle's topology fingerprint (CPU only).

The paper (Section 4.2.1, Section 5.3) only requires that equal keys mean equal topology.
Pins: the published SplitMix64 test vector for `mix`; grouping equal to exact equality of
the masked node sequences; a closed-form power-sum evaluation in Python integers; mutants
(swap / truncate / append / field change) change the key; template counts of the configs.
"""
import os

import numpy as np
import pytest

from synth import layout as L
from tests.cases import small

M64 = (1 << 64) - 1
P = 0x9E3779B97F4A7C15
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_seed1234567.txt")


def test_mix_matches_published_splitmix64_vector(oracle):
    want = [int(l) for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(want) == 5
    state = 1234567
    for w in want:
        state = (state + P) & M64
        assert oracle.mix(state) == w


def py_node_hash(n, mask, mix):
    kid = int(n["kernel_id"]) if mask & L.FP_KERNEL_ID else 0
    g = [int(x) for x in n["grid"]]
    b = [int(x) for x in n["block"]]
    for c, bit in enumerate((L.FP_GRID_X, L.FP_GRID_Y, L.FP_GRID_Z)):
        if not mask & bit:
            g[c] = 0
    if not mask & L.FP_BLOCK:
        b = [0, 0, 0]
    ln = int(n["blob_len"]) if mask & L.FP_BLOB_LEN else 0
    fl = int(n["flags"]) if mask & L.FP_FLAGS else 0
    a = mix((kid + P) & M64)
    a = mix(a ^ (g[0] | g[1] << 32))
    a = mix(a ^ (g[2] | b[0] << 32))
    a = mix(a ^ (b[1] | b[2] << 32))
    a = mix(a ^ (ln | fl << 32))
    return a


@pytest.mark.parametrize("idx,mask", [(1, L.FP_ALL), (2, L.FP_ALL & ~L.FP_GRID_X), (2, L.FP_ALL)])
def test_key_equals_closed_form_power_sum_in_python_integers(oracle, idx, mask):
    ar = small(idx)
    keys, _, _ = oracle.fingerprint(ar.nodes, ar.node_off, mask)
    for g in range(min(ar.n_graphs, 3)):
        nodes = ar.nodes[int(ar.node_off[g]):int(ar.node_off[g + 1])]
        N = len(nodes)
        total = oracle.mix(N) * pow(P, N, 1 << 64)
        for n, nd in enumerate(nodes):
            total += py_node_hash(nd, mask, oracle.mix) * pow(P, N - 1 - n, 1 << 64)
        assert keys[g] == oracle.mix(total & M64)
    assert np.array_equal(keys, oracle.fingerprint_powersum(ar.nodes, ar.node_off, mask))


@pytest.mark.parametrize("idx", [1, 2, 3, 5])
def test_grouping_equals_exact_sequence_equality(oracle, idx):
    ar = small(idx)
    for mask in (ar.fp_mask, L.FP_ALL, L.FP_KERNEL_ID | L.FP_BLOB_LEN):
        keys, tid, tg = oracle.fingerprint(ar.nodes, ar.node_off, mask)
        etid, etg = oracle.group_exact(ar.nodes, ar.node_off, mask)
        assert np.array_equal(tid, etid) and np.array_equal(tg, etg)
        # equal ids <=> equal keys
        for t, g0 in enumerate(tg):
            assert np.all(keys[tid == t] == keys[g0])
            assert tid[g0] == t and (tid[:g0] != t).all()
        assert len(set(keys.tolist())) == len(tg)
    # under the config's mask the grouping is the generator's construction
    _, tid, tg = oracle.fingerprint(ar.nodes, ar.node_off, ar.fp_mask)
    assert np.array_equal(tid, ar.graph_tmpl) and np.array_equal(tg, ar.tmpl_graph)
    assert len(tg) <= 3


def test_full_mask_separates_graphs_with_different_grids(oracle):
    ar = small(2)
    _, tid, tg = oracle.fingerprint(ar.nodes, ar.node_off, L.FP_ALL)
    # batch sizes 1, 2, 8, 16 give the same ceil(bs/16) grid; the others differ
    assert len(tg) > ar.n_templates


def test_mutants_change_the_key(oracle):
    ar = small(1)
    nodes = ar.nodes.copy()
    N = len(nodes)

    def key(nd):
        return oracle.fingerprint(nd, np.array([0, len(nd)], np.uint64), L.FP_ALL)[0][0]

    k0 = key(nodes)
    assert key(nodes.copy()) == k0
    sw = nodes.copy()
    sw[[3, 4]] = sw[[4, 3]]
    assert key(sw) != k0  # order-sensitive
    assert key(nodes[:-1]) != k0 and key(nodes[1:]) != k0  # truncation
    assert key(np.concatenate([nodes, nodes[:1]])) != k0  # append
    for fld, sub in (("kernel_id", None), ("grid", 0), ("grid", 1), ("grid", 2), ("block", 0),
                     ("block", 1), ("block", 2), ("blob_len", None), ("flags", None)):
        mu = nodes.copy()
        if sub is None:
            mu[fld][N // 2] += 1
        else:
            mu[fld][N // 2, sub] += 1
        assert key(mu) != k0, fld
    # a masked-out field does not matter, every other field still does
    mask = L.FP_ALL & ~L.FP_GRID_X

    def keym(nd):
        return oracle.fingerprint(nd, np.array([0, len(nd)], np.uint64), mask)[0][0]

    mu = nodes.copy()
    mu["grid"][:, 0] += 5
    assert keym(mu) == keym(nodes)
    mu["grid"][7, 1] += 1
    assert keym(mu) != keym(nodes)
    # swapping values between the two halves of a packed word changes the key
    a = nodes[:1].copy()
    b = a.copy()
    b["grid"][0, 0], b["grid"][0, 1] = a["grid"][0, 1], a["grid"][0, 0]
    if a["grid"][0, 0] != a["grid"][0, 1]:
        assert key(a) != key(b)


def test_empty_graphs_and_length_salt(oracle):
    nodes = np.zeros(3, L.NODE)
    off = np.array([0, 0, 1, 3, 3], np.uint64)  # lengths 0, 1, 2, 0
    keys, tid, tg = oracle.fingerprint(nodes, off, L.FP_ALL)
    assert keys[0] == keys[3] == oracle.mix(oracle.mix(0))
    assert len({int(k) for k in keys}) == 3
    assert tid.tolist() == [0, 1, 2, 0] and tg.tolist() == [0, 1, 2]
