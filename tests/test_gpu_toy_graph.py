"""Tiny end-to-end check: materialized argument words installed into an executable hipGraph
of toy kernels with hipGraphExecKernelNodeSetParams, graph replayed (the on-demand update of
Section 4.2.1 / Section 5.3, with arguments produced by the library)."""
import ctypes as C
import os

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "toy_graph", "libtoy_graph.so")


def test_toy_graph_install_and_replay():
    import torch

    assert torch.cuda.is_available()
    assert os.path.exists(LIB), "build it first: python -c 'import __graft_entry__ as g; g.build()'"
    import paper_2604_06664_amd as fdy

    fdy.lib()  # libfdy.so is loaded first; the toy library resolves its fdy_* symbols against it
    C.CDLL(fdy.LIB_PATH, mode=C.RTLD_GLOBAL)
    toy = C.CDLL(LIB)
    toy.toy_graph_check.restype = C.c_int
    toy.toy_graph_check.argtypes = [C.c_char_p, C.c_int]
    msg = C.create_string_buffer(512)
    print("[toy] hipGraph install + replay", flush=True)
    rc = toy.toy_graph_check(msg, 512)
    print("[toy]", msg.value.decode(), flush=True)
    assert rc == 0, msg.value.decode()
