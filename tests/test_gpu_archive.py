"""The binary archive end to end on the GPU: SAVE side (scan, segmentation, fingerprint run on
the device, results written to a file), LOAD side (open, verify, check, one copy to a device
slab, materialize straight from the slab's sections), compared with the oracle's materialize
of the same archive.  Needs a real MI355X (`-m gpu`)."""
import time

import numpy as np
import pytest

from synth import MatProblem, make_config
from synth import layout as L
from synth.sections import archive_sections
from tests.cases import small

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def hip():
    import torch

    assert torch.cuda.is_available(), "gpu tests need a GPU"
    import paper_2604_06664_amd as fdy
    from tests.support import session

    fdy.lib()
    return session


def save_side(hip, ar):
    """Relocations, their per-graph offsets and the topology keys, computed on the device."""
    import torch

    import paper_2604_06664_amd as fdy

    G = ar.n_graphs
    run = hip.ScanRun(ar.words, ar.table)
    run.launch()
    d_word_off = fdy.to_device(ar.word_off)
    d_reloc_off = fdy.device_bytes((G + 1) * 8, fill=0xEE)
    fdy.fdy_reloc_segment(run.d_relocs, run.d_count, run.capacity, d_word_off, G + 1, d_reloc_off)
    d_keys = fdy.device_bytes(G * 8, fill=0xEE)
    d_tid = fdy.device_bytes(G * 4, fill=0xEE)
    d_tg = fdy.device_bytes(G * 4, fill=0xEE)
    d_nt = torch.full((1,), -1, dtype=torch.int32, device="cuda:0")
    fdy.fdy_fingerprint(fdy.to_device(ar.nodes), fdy.to_device(ar.node_off), G, ar.fp_mask, d_keys, d_tid, d_tg,
                        d_nt)
    relocs, count, status = run.result()
    assert status == 0 and count == len(relocs)
    # the generator's manifest is the one the device finds
    assert int(d_nt.item()) == ar.n_templates
    assert np.array_equal(fdy.to_host(d_tid, np.uint32, G), ar.graph_tmpl)
    assert np.array_equal(fdy.to_host(d_tg, np.uint32, ar.n_templates), ar.tmpl_graph)
    return relocs, fdy.to_host(d_reloc_off, np.uint64, G + 1), fdy.to_host(d_keys, np.uint64, G)


@pytest.mark.parametrize("idx,compact", [(2, False), (2, True), (3, False), (3, True), (5, True)])
def test_archive_file_to_materialized_blobs(hip, oracle, tmp_path, idx, compact):
    import torch

    import paper_2604_06664_amd as fdy
    from paper_2604_06664_amd import archive as A

    ar = small(idx)
    say(f"[archive] {ar.name} compact={compact} G={ar.n_graphs} M={ar.n_maps}")
    relocs, reloc_off, keys = save_side(hip, ar)
    path = tmp_path / "a.fdya"
    A.fdy_archive_write(path, archive_sections(ar, relocs, reloc_off, keys=keys, compact=compact))

    h = A.fdy_archive_open(path, A.FDY_ARCHIVE_VERIFY_SUMS)
    try:
        info = A.fdy_archive_check(h)
        assert info.n_graphs == ar.n_graphs and info.n_templates == ar.n_templates
        assert info.n_src_graphs == (ar.n_templates if compact else ar.n_graphs)
        nbytes = A.fdy_archive_body_bytes(h)
        d_slab = fdy.device_bytes(nbytes, fill=0xEE)
        A.fdy_archive_upload(h, d_slab, nbytes)
        torch.cuda.synchronize()
        desc = A.fdy_archive_mat_desc(h, d_slab)
    finally:
        A.fdy_archive_close(h)  # the slab is self-contained once the copy is done

    d_new_base = fdy.to_device(np.ascontiguousarray(ar.new_base, np.uint64))
    d_map_rank = None if ar.map_rank is None else fdy.to_device(np.ascontiguousarray(ar.map_rank, np.uint32))
    desc.n_maps = ar.n_maps
    desc.new_base = d_new_base.data_ptr()
    desc.map_rank = None if d_map_rank is None else d_map_rank.data_ptr()
    if d_map_rank is None:
        desc.n_ranks = 0
    wpm, nt = desc.out_words_per_map, desc.out_nodes_total
    d_out = fdy.device_bytes(ar.n_maps * wpm * 8, fill=0xCD)
    d_dims = fdy.device_bytes(nt * 24, fill=0xCD)
    ws = fdy.fdy_materialize_workspace_bytes(desc)
    d_ws = fdy.device_bytes(ws)
    d_status = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    fdy.fdy_materialize(desc, d_out, d_dims, d_ws, ws, d_status)
    torch.cuda.synchronize()
    assert int(d_status.item()) == 0
    out = fdy.to_host(d_out, np.uint64, ar.n_maps * wpm).reshape(ar.n_maps, wpm)
    dims = fdy.to_host(d_dims, np.uint32, nt * 6).reshape(-1, 6)

    # the oracle's side never sees the file: the synthetic archive, scanned by the oracle
    orelocs, _ = oracle.scan(ar.words, ar.table)
    mp = MatProblem.from_archive(ar, orelocs, oracle.reloc_segment(orelocs, ar.word_off))
    ref, rdims = oracle.materialize(mp, True)
    assert np.array_equal(out, ref)
    assert np.array_equal(dims, rdims)


def test_archive_load_time_full_moe_decode(hip, oracle, tmp_path):
    """Config 3 at full size (67 graphs of 2632 nodes, 8 ranks): file -> device-resident,
    checked archive; host times are printed for the record."""
    import torch

    import paper_2604_06664_amd as fdy
    from paper_2604_06664_amd import archive as A

    ar = make_config(3)
    relocs, reloc_off, keys = save_side(hip, ar)
    path = tmp_path / "moe.fdya"
    A.fdy_archive_write(path, archive_sections(ar, relocs, reloc_off, keys=keys))
    t0 = time.perf_counter()
    h = A.fdy_archive_open(path, A.FDY_ARCHIVE_VERIFY_SUMS)
    t1 = time.perf_counter()
    info = A.fdy_archive_check(h)
    t2 = time.perf_counter()
    nbytes = A.fdy_archive_body_bytes(h)
    d_slab = fdy.device_bytes(nbytes)
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    A.fdy_archive_upload(h, d_slab, nbytes)
    torch.cuda.synchronize()
    t4 = time.perf_counter()
    say(f"[archive] moe_decode {nbytes / 1e6:.1f} MB: open+sums {1e3 * (t1 - t0):.2f} ms, check "
        f"{1e3 * (t2 - t1):.2f} ms, upload {1e3 * (t4 - t3):.2f} ms ({nbytes / (t4 - t3) / 1e9:.1f} GB/s)")
    assert info.n_graphs == ar.n_graphs and info.n_relocs == len(relocs)
    # the slab holds the file's body bit for bit
    for kind, arr in archive_sections(ar, relocs, reloc_off, keys=keys):
        raw = np.ascontiguousarray(arr).view(np.uint8).reshape(-1)
        p = A.fdy_archive_device_section(h, kind, d_slab)
        off = p - d_slab.data_ptr()
        assert np.array_equal(d_slab[off: off + raw.size].cpu().numpy(), raw)
    A.fdy_archive_close(h)
    assert (t2 - t0) < 0.1
