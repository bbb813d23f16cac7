"""The whole hot path captured into a HIP graph and replayed (GPU).

Every entry point only enqueues kernels on the caller's stream, so a step can be captured
once and replayed; this checks it: capture scan -> segmentation -> fingerprint ->
materialize (and the fused scan + rebase, and the scan at 4-byte stride) on a side stream, then replay several times with
outputs poisoned and eager work of the same library between the replays, and compare every
replay with the eager result bit for bit."""
import numpy as np
import pytest

from tests.cases import small

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("idx,own_tiles", [(2, True), (3, True), (3, False)])
def test_captured_step_replays_like_eager(idx, own_tiles):
    """own_tiles False: the materialization is captured in its form with a prep launch (which
    inputs this small would not take by themselves)."""
    import torch

    assert torch.cuda.is_available()
    import paper_2604_06664_amd as fdy

    fdy.lib()
    default_limit = fdy.tune_get(fdy.TUNE_MAT_SELF_WGS)
    if not own_tiles:
        fdy.tune_set(fdy.TUNE_MAT_SELF_WGS, 0)
    try:
        _capture_and_replay(idx)
    finally:
        fdy.tune_set(fdy.TUNE_MAT_SELF_WGS, default_limit)


def _capture_and_replay(idx):
    import torch

    import paper_2604_06664_amd as fdy
    from tests.support import session

    ar = small(idx)
    run = session.PathRun(ar, reloc_capacity=len(ar.ptr_word) + 64)
    fused = session.ScanRebaseRun(ar.words, ar.table, ar.new_base[0])
    units = np.ascontiguousarray(ar.words).view(np.uint32)
    s4 = session.ScanStride4Run(units, ar.table)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        run.step(side)
        fused.launch(side)
        s4.launch(side)
    torch.cuda.synchronize()
    assert run.status() == 0
    ref_out = run.mat.d_out.clone()
    ref_relocs = run.scan.d_relocs.clone()
    ref_count = int(run.scan.d_count.item())
    ref_fused = fused.d_out.clone()
    assert ref_count == len(ar.ptr_word)
    ref_s4 = s4.d_relocs.clone()
    ref_s4_count = int(s4.d_count.item())
    assert ref_s4_count >= ref_count and int(s4.d_status.item()) == 0

    print(f"[graph] capture config {idx}", flush=True)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run.step(side)
        fused.launch(side)
        s4.launch(side)
    torch.cuda.synchronize()

    other = session.ScanRun(ar.words[: len(ar.words) // 2], ar.table)  # eager work between replays
    for rep in range(4):
        run.mat.d_out.fill_(0xCD)
        run.scan.d_relocs.fill_(0xCD)
        run.scan.d_count.fill_(-1)
        fused.d_out.fill_(0xCD)
        fused.d_count.fill_(-1)
        s4.d_relocs.fill_(0xCD)
        s4.d_count.fill_(-1)
        other.launch()
        torch.cuda.synchronize()
        print(f"[graph] replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert int(run.scan.d_count.item()) == ref_count and run.status() == 0
        assert torch.equal(run.scan.d_relocs[: ref_count * 16], ref_relocs[: ref_count * 16])
        assert torch.equal(run.mat.d_out, ref_out)
        assert int(fused.d_count.item()) == ref_count
        assert torch.equal(fused.d_out, ref_fused)
        assert int(s4.d_count.item()) == ref_s4_count and int(s4.d_status.item()) == 0
        assert torch.equal(s4.d_relocs[: ref_s4_count * 16], ref_s4[: ref_s4_count * 16])
        _, cnt, st = other.result()
        assert st == 0 and cnt > 0
