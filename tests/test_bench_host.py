"""Host-side logic of bench.py that needs no GPU: the refusal of more than one GPU, the byte
accounting behind the roofline figures, and the parser that takes the measured memory traffic
from the committed rocprofv3 summaries."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from tests.cases import small  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_are_each_distinct_byte_once():
    """Worked by hand on a small archive: words in, relocation entries out, table in (scan);
    template words, their relocation entries, base maps, lists in and every output word out
    (materialize); words in and out, relocation entries, table and one base map (scan with
    output).  Config 4's figures at full size follow from the same formulas:
    2^27*16 + 13,423,977*16 + 2^20*24 = 2,387,433,104 for the scan with output."""
    ar = small(2)
    n_rel, n_rel_tmpl = 1000, 300
    b = bench.algorithmic_bytes(ar, n_rel, n_rel_tmpl)
    W, A, M = len(ar.words), ar.n_alloc, ar.n_maps
    nw = np.diff(ar.word_off.astype(np.int64))
    tmpl_words = sum(int(nw[g]) for g in ar.tmpl_graph)
    out_words = sum(int(nw[ar.tmpl_graph[t]]) for t in ar.graph_tmpl) * M
    assert b["scan"] == 8 * W + 16 * n_rel + 16 * A
    assert b["mat"] == 8 * tmpl_words + 16 * n_rel_tmpl + 8 * M * A + ar.ovr.nbytes + ar.patch.nbytes + 8 * out_words
    assert b["scan_out"] == 16 * W + 16 * n_rel + 24 * A
    assert b["in_blob"] == 8 * W and b["out_blob"] == 8 * out_words
    assert (2 ** 27) * 16 + 13_423_977 * 16 + (2 ** 20) * 24 == 2_387_433_104


def test_traffic_comes_from_the_committed_summaries(tmp_path, monkeypatch):
    # what the committed profiles hold for the headline kernel: a plausible figure, at least the
    # algorithmic bytes and below three times that
    t = bench.pmc_traffic_bytes(4, "scan_out_kernel")
    assert t is not None and 2_387_433_104 <= t < 3 * 2_387_433_104
    assert bench.pmc_traffic_bytes(4, "no_such_kernel") is None
    assert bench.pmc_traffic_bytes(99, "scan_out_kernel") is None
    # the parser itself, on a file of its own
    prof = tmp_path / "profiles"
    prof.mkdir()
    (prof / "x.txt").write_text("some text\n  traffic: workload=7 kernel=k_a fetch_bytes=100 write_bytes=23\n"
                                "traffic: workload=7 kernel=k_b fetch_bytes=1 write_bytes=2 trailing words\n"
                                "traffic: workload=7 kernel=k_c fetch_bytes=x write_bytes=2\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.pmc_traffic_bytes(7, "k_a") == 123
    assert bench.pmc_traffic_bytes(7, "k_b") == 3
    assert bench.pmc_traffic_bytes(7, "k_c") is None
    assert bench.pmc_traffic_bytes(8, "k_a") is None
