"""fdy_materialize_static (the entry point that allocates nothing: its per-call tables lie in a
fixed array inside the library) against fdy_materialize, through the C-ABI: bit-equal outputs
on two calls in a row, the second with a smaller input.  Collected last on purpose."""
import numpy as np
import pytest

from synth import MatProblem, make_config
from tests.cases import small

pytestmark = pytest.mark.gpu


def _problem(oracle, ar, **kw):
    relocs, _ = oracle.scan(ar.words, ar.table)
    return MatProblem.from_archive(ar, relocs, oracle.reloc_segment(relocs, ar.word_off), **kw)


def test_materialize_static_equals_materialize(oracle):
    import torch

    assert torch.cuda.is_available()
    import paper_2604_06664_amd as fdy
    from tests.support import session

    fdy.lib()
    assert fdy.fdy_materialize_static_limit() == 4 << 20
    # first the larger input (MoE shape: 8 rank maps, patches, launch dimensions), then a smaller
    # one (dense shape), then the larger again: the scratch keeps the last call's contents
    tiny = make_config(2, layers=2, batch_sizes=[1, 16, 136])  # 3 graphs of 32 nodes
    cases = [_problem(oracle, small(3)), _problem(oracle, tiny), _problem(oracle, small(3))]
    assert cases[1].out_words_per_map() * cases[1].M < cases[0].out_words_per_map() * cases[0].M // 8
    # Launches this small would resolve their tiles inside the main kernel and leave the scratch
    # alone: the knob that decides it is set to "never" first, so that the tile tables really
    # lie in the library's array, and to its default afterwards.
    default_limit = fdy.tune_get(fdy.TUNE_MAT_SELF_WGS)
    try:
        for self_wgs in (0, default_limit):
            fdy.tune_set(fdy.TUNE_MAT_SELF_WGS, self_wgs)
            for n, mp in enumerate(cases):
                print(f"[no-alloc] self-resolving up to {self_wgs} workgroups, call {n}: G={mp.G} M={mp.M} "
                      f"words/map={mp.out_words_per_map()}", flush=True)
                ref_run = session.MatRun(mp)
                ref_run.launch()
                ref_out, ref_dims, ref_status = ref_run.result()
                assert ref_status == 0
                run = session.MatRun(mp)  # same uploads and descriptor; its workspace stays unused
                assert fdy.fdy_materialize_workspace_bytes(run.desc) <= fdy.fdy_materialize_static_limit()
                fdy.fdy_materialize_static(run.desc, run.d_out, run.d_dims, run.d_status)
                out, dims, status = run.result()
                assert status == 0
                assert np.array_equal(out, ref_out) and np.array_equal(dims, ref_dims)
                want, want_dims = oracle.materialize(mp)
                assert np.array_equal(out, want) and np.array_equal(dims, want_dims)
    finally:
        fdy.tune_set(fdy.TUNE_MAT_SELF_WGS, default_limit)
    # a descriptor beyond the fixed scratch is refused on the host, nothing is launched
    big = session.MatRun(cases[0])
    big.desc.out_words_per_map = 1 << 39
    assert fdy.fdy_materialize_workspace_bytes(big.desc) > fdy.fdy_materialize_static_limit()
    rc = fdy.fdy_materialize_static(big.desc, big.d_out, big.d_dims, big.d_status, check=False)
    assert rc == fdy.FDY_ERR_WORKSPACE
