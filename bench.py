#!/usr/bin/env python3
"""bench.py - one-GPU throughput of the whole hot path (scan -> reloc segmentation ->
fingerprint -> materialize) on the synthetic capture archives, with the roofline fraction of
the dominant kernel and the CPU oracle timed beside it.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 4] [--no-others]

Prints ONE JSON line.  `value` is param-blob GB/s for scan+materialize on the main workload
(config 4, the largest single-GPU configuration): (input blob bytes + output blob bytes) per
step time, inputs resident in HBM.  A step is one pass of the whole path over the archive:
the allocation table's search hierarchy is prepared once per archive, outside the step (the
layout is fixed for the life of an archive), everything else runs in every step.  An archive
whose graphs are their own templates, with one base map and nothing to override or patch
(config 4), takes the path in which the scan writes the materialized output itself
(fdy_scan_pointers_rebase); the two-call path on the same archive is reported beside it.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak



def pmc_traffic_bytes(workload, kernel):
    """Memory-side traffic per launch in bytes (read + write) of `kernel` on `workload`, from the
    committed rocprofv3 summaries under profiles/: FETCH_SIZE and WRITE_SIZE of two separate
    counter runs of this script, each scaled by what the same counter reads for a plain 1 GiB
    device copy in the same run.  A counter run cannot happen inside this process, so the
    figures are read from the summaries' machine-readable lines
        traffic: workload=<n> kernel=<name> fetch_bytes=<int> write_bytes=<int>
    and are None for workloads and kernels that no summary covers."""
    import glob
    import re

    pat = re.compile(r"^traffic:\s+workload=(\d+)\s+kernel=(\S+)\s+fetch_bytes=(\d+)\s+write_bytes=(\d+)")
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        with open(path) as f:
            for line in f:
                m = pat.match(line.strip())
                if m and int(m.group(1)) == workload and m.group(2) == kernel:
                    return int(m.group(3)) + int(m.group(4))
    return None


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def algorithmic_bytes(ar, n_relocs_total, n_relocs_tmpl):
    """Compulsory HBM bytes per launch of the two streaming kernels: every distinct input
    byte once plus every output byte once (re-reads of templates per map are not counted)."""
    W, A, M = len(ar.words), ar.n_alloc, ar.n_maps
    import numpy as np

    nw = np.diff(ar.word_off.astype(np.int64))
    tmpl_words = int(nw[ar.tmpl_graph].sum())
    out_words = int(nw[ar.tmpl_graph[ar.graph_tmpl]].sum()) * M
    scan = W * 8 + n_relocs_total * 16 + A * 16
    mat = (tmpl_words * 8 + n_relocs_tmpl * 16 + M * A * 8 + ar.ovr.nbytes + ar.patch.nbytes
           + out_words * 8)
    # the scan that also writes the rebased output: words in, words out, table, one base map
    scan_out = W * 16 + n_relocs_total * 16 + A * 16 + A * 8
    return dict(scan=scan, mat=mat, scan_out=scan_out, in_blob=W * 8, out_blob=out_words * 8,
                out_words=out_words)


ALG_OF = {"scan_kernel": "scan", "mat_main_kernel": "mat", "scan_out_kernel": "scan_out"}


def run_workload(idx, steps, warmup, prof=True, cpu_sample_words=0, timed_events=True, label=None,
                 one_pass=None, two_call_too=False, **config_kw):
    import numpy as np
    import torch

    import paper_2604_06664_amd as fdy
    from tests.support import session
    from synth import CONFIG_NAMES, make_config

    t0 = time.time()
    ar = make_config(idx, **config_kw)
    label = label or f"config {idx}: {CONFIG_NAMES[idx]}"
    log(f"{label}: generated in {time.time() - t0:.1f}s "
        f"W={len(ar.words)} A={ar.n_alloc} G={ar.n_graphs} M={ar.n_maps} T={ar.n_templates}")
    n_ptr = len(ar.ptr_word)
    run = session.PathRun(ar, reloc_capacity=n_ptr + 1024, one_pass=one_pass)
    stream = torch.cuda.current_stream()
    for _ in range(max(warmup, 1)):
        run.step(stream)
    st = run.status()
    cnt = int(run.scan.d_count.item())
    assert st == 0 and cnt == n_ptr, f"status={st} count={cnt} planted={n_ptr}"
    # timed region: exactly `steps` steps; only the two streaming kernels are bracketed by events
    # (an event pair costs a few microseconds: the launch-bound secondary workloads are timed
    # without any, their kernel times all come from the untimed pass below)
    if prof and timed_events:
        fdy.prof_enable(steps, slots=(fdy.PROF_SCAN_MAIN, fdy.PROF_MAT_MAIN, fdy.PROF_SCAN_OUT))
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(steps):
        run.step(stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    dev_ms = ev0.elapsed_time(ev1)
    kernels = fdy.prof_read() if prof and timed_events else {}
    # untimed extra pass: every kernel bracketed, for the breakdown
    if prof:
        fdy.prof_enable(steps)
        for _ in range(steps):
            run.step(stream)
        torch.cuda.synchronize()
        for name, k in fdy.prof_read().items():
            kernels.setdefault(name, k)
        fdy.prof_enable(0)
    assert run.status() == 0
    # relocs belonging to template graphs (what materialize reads)
    roff = fdy.to_host(run.d_reloc_off, np.uint64, ar.n_graphs + 1).astype(np.int64)
    n_rel_tmpl = int((roff[1:] - roff[:-1])[ar.tmpl_graph].sum())
    ab = algorithmic_bytes(ar, cnt, n_rel_tmpl)
    ms = wall_ms / steps
    step_calls = ("fdy_scan_pointers_rebase + fdy_segment_fingerprint" if run.one_pass else
                  "fdy_scan_pointers + fdy_segment_fingerprint + fdy_materialize")
    res = dict(
        workload=label, step=step_calls + " (table prepared once per archive)",
        ms_per_step=ms, device_ms_per_step=dev_ms / steps,
        blob_gbs=(ab["in_blob"] + ab["out_blob"]) / ms / 1e6,
        graphs_per_s=ar.n_graphs * ar.n_maps / (ms / 1e3),
        words=len(ar.words), allocations=ar.n_alloc, graphs=ar.n_graphs, maps=ar.n_maps,
        templates=ar.n_templates, relocs=cnt, out_bytes=ab["out_blob"], kernels={})
    for name, k in kernels.items():
        e = dict(avg_ms=round(k["avg_ms"], 5), min_ms=round(k["min_ms"], 5), n=k["n"])
        alg = ab[ALG_OF[name]] if name in ALG_OF else None
        if alg is not None:
            e["algorithmic_bytes"] = alg
            e["achieved_gbs"] = round(alg / k["avg_ms"] / 1e6, 1)
            e["frac_hbm_peak"] = round(alg / k["avg_ms"] / 1e6 / HBM_PEAK_GBS, 4)
        res["kernels"][name] = e
    res["launches_per_step"] = len(res["kernels"])
    res["algorithmic_bytes_per_step"] = sum(e.get("algorithmic_bytes", 0) for e in res["kernels"].values())
    res["frac_hbm_peak_step"] = round(res["algorithmic_bytes_per_step"] / ms / 1e6 / HBM_PEAK_GBS, 4)
    if res["kernels"].get("mat_main_kernel"):
        res["materialize_graphs_per_s"] = ar.n_graphs * ar.n_maps / (
            res["kernels"]["mat_main_kernel"]["avg_ms"] / 1e3)
    if ar.n_graphs == 1 and ar.n_maps == 1 and prof and two_call_too:
        res["fused_scan_rebase"] = fused_variant(ar, run, steps)
    if two_call_too and run.one_pass:
        res["two_call_path"] = two_call_path(ar, run, steps)
    if len(ar.words) < (1 << 24):  # launch-bound sizes: the same step replayed from a HIP graph
        res["graph_replay"] = graph_replay(run, steps)
    cpu = None
    if cpu_sample_words:
        cpu = cpu_baseline(ar, run, min(cpu_sample_words, len(ar.words)))
    del run
    torch.cuda.empty_cache()
    return res, cpu


def two_call_path(ar, one, steps):
    """The same archive through fdy_scan_pointers + fdy_materialize (the words read twice):
    beside the step, never part of `value`.  Its outputs must equal the one-pass step's."""
    import torch

    import paper_2604_06664_amd as fdy
    from tests.support import session

    run = session.PathRun(ar, reloc_capacity=one.scan.capacity, one_pass=False)
    stream = torch.cuda.current_stream()
    for _ in range(2):
        run.step(stream)
    assert run.status() == 0
    fdy.prof_enable(steps, slots=(fdy.PROF_SCAN_MAIN, fdy.PROF_MAT_MAIN))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run.step(stream)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    k = fdy.prof_read()
    fdy.prof_enable(0)
    n = int(run.scan.d_count.item())
    same = (bool(torch.equal(run.mat.d_out, one.mat.d_out)) and n == int(one.scan.d_count.item())
            and bool(torch.equal(run.scan.d_relocs[: n * 16], one.scan.d_relocs[: n * 16])))
    out = dict(ms_per_step=round(ms, 4), scan_kernel_avg_ms=round(k["scan_kernel"]["avg_ms"], 5),
               mat_main_kernel_avg_ms=round(k["mat_main_kernel"]["avg_ms"], 5), equals_one_pass_outputs=same)
    del run
    torch.cuda.empty_cache()
    return out


def graph_replay(run, steps):
    """The step captured once into a HIP graph and replayed: for the small archives the eager
    step is bound by launch latency (eight launches of 5-20 us), which a graph removes.  Not
    part of `value`.  The replayed output must equal the eager one."""
    import torch

    try:
        ref = run.mat.d_out.clone()
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            run.step(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            run.step(side)
        torch.cuda.synchronize()
        run.mat.d_out.fill_(0xCD)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        same = bool(torch.equal(run.mat.d_out, ref)) and run.status() == 0
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(steps):
            graph.replay()
        ev1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        return dict(ms_per_step=round(wall, 5), device_ms_per_step=round(ev0.elapsed_time(ev1) / steps, 5),
                    equals_eager_output=same)
    except Exception as e:  # reported, never fatal for the bench line
        return dict(error=f"{type(e).__name__}: {e}")


def fused_variant(ar, run, steps):
    """The one-pass variant (fdy_scan_rebase) on the same archive: not part of the step that
    `value` times, reported beside it.  Its output must equal the two-call path's."""
    import torch

    import paper_2604_06664_amd as fdy
    from tests.support import session

    fr = session.ScanRebaseRun(run.scan.d_words, run.scan.d_table, ar.new_base[0],
                               n_words=len(ar.words), n_alloc=ar.n_alloc)
    stream = torch.cuda.current_stream()
    for _ in range(2):
        fr.launch(stream)
    fdy.prof_enable(steps, slots=(fdy.PROF_SCAN_REBASE,))
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record(stream)
    for _ in range(steps):
        fr.launch(stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    k = fdy.prof_read()["scan_rebase_kernel"]
    fdy.prof_enable(0)
    ms = ev0.elapsed_time(ev1) / steps
    W = len(ar.words)
    alg = W * 16 + ar.n_alloc * 24
    same = bool(torch.equal(fr.d_out[: W * 8], run.mat.d_out[: W * 8]))
    out = dict(ms_per_call=round(ms, 4), blob_gbs=round(2 * W * 8 / ms / 1e6, 1),
               kernel_avg_ms=round(k["avg_ms"], 5), algorithmic_bytes=alg,
               frac_hbm_peak=round(alg / k["avg_ms"] / 1e6 / HBM_PEAK_GBS, 4),
               equals_two_call_output=same)
    del fr
    return out


def cpu_baseline(ar, run, n):
    """The oracle as it stands, single thread, on the first n words of the same workload:
    scan + segmentation + materialize (one map).  Also checks the GPU relocation table of
    that prefix against the oracle's."""
    import numpy as np

    import oracle
    import paper_2604_06664_amd as fdy
    from synth import MatProblem

    oracle.build()
    words = ar.words[:n]
    t0 = time.perf_counter()
    relocs, cnt = oracle.scan(words, ar.table)
    t_scan = time.perf_counter() - t0
    woff = np.array([0, n], np.uint64)
    t0 = time.perf_counter()
    roff = oracle.reloc_segment(relocs, woff)
    mp = MatProblem(
        src_words=words, src_word_off=woff, src_nodes=ar.nodes[:0], src_node_off=[0, 0], relocs=relocs,
        src_reloc_off=roff, tmpl_graph=[0], graph_tmpl=[0], ovr=ar.ovr[:0], ovr_off=[0, 0],
        govr=ar.govr[:0], govr_off=[0, 0], new_base=ar.new_base[:1], map_rank=None, n_ranks=0,
        patch=ar.patch[:0], patch_off=[0])
    out, _ = oracle.materialize(mp, want_dims=False)
    t_mat = time.perf_counter() - t0
    got = fdy.to_host(run.scan.d_relocs, session_reloc_dtype(), cnt)
    parity = bool(np.array_equal(got, relocs))
    got_out = fdy.to_host(run.mat.d_out, np.uint64, n)
    parity = parity and bool(np.array_equal(got_out, out[0]))
    secs = t_scan + t_mat
    # secondary: the same oracle scan function over disjoint word ranges on all host cores (the
    # paper's preparation "scales linearly with CPU threads", Section 4.2.1); no new logic
    from concurrent.futures import ThreadPoolExecutor

    threads = min(16, os.cpu_count() or 1)
    cuts = [n * i // threads for i in range(threads + 1)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(lambda i: oracle.scan(words[cuts[i]:cuts[i + 1]], ar.table)[1], range(threads)))
    t_scan_mt = time.perf_counter() - t0
    mt_ok = sum(parts) == cnt
    return dict(value=round(2 * n * 8 / secs / 1e9, 4), unit="GB/s", cores=1, kind="oracle",
                sample=f"first {n} words ({n * 8 / 2**20:.0f} MiB) of the workload against the full "
                       f"allocation table: scan {t_scan:.2f}s + segment+materialize {t_mat:.2f}s, "
                       f"single thread",
                scan_gbs=round(n * 8 / t_scan / 1e9, 4), materialize_gbs=round(n * 8 / t_mat / 1e9, 4),
                gpu_matches_oracle_on_sample=parity,
                all_cores=dict(value=round(2 * n * 8 / (t_scan_mt + t_mat) / 1e9, 4), unit="GB/s",
                               cores=threads, scan_s=round(t_scan_mt, 3), counts_agree=mt_ok,
                               note="oracle scan over disjoint word ranges, one range per thread; "
                                    "materialize single-threaded"))


def session_reloc_dtype():
    from tests.support import session

    return session.RELOC


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=4, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--cpu-sample-words", type=int, default=1 << 27)
    ap.add_argument("--no-others", action="store_true", help="skip the secondary configurations")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known HBM traffic, "
                         "used to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (every unit of the hot path is "
              "independent, so ranks would run it without communication) - run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    import paper_2604_06664_amd as fdy

    fdy.lib()
    if args.calibrate_copy:
        a = torch.zeros(1 << 27, dtype=torch.int64, device="cuda:0")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    main_res, cpu = run_workload(args.workload, args.steps, args.warmup, prof=True,
                                 cpu_sample_words=args.cpu_sample_words, two_call_too=True)
    k = main_res["kernels"]
    dom = max((n for n in k if "algorithmic_bytes" in k[n]), key=lambda n: k[n]["avg_ms"])
    roofline = dict(bound="hbm", kernel=dom, achieved=k[dom]["achieved_gbs"], peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=k[dom]["frac_hbm_peak"],
                    traffic=pmc_traffic_bytes(args.workload, dom),
                    algorithmic_bytes_per_launch=k[dom]["algorithmic_bytes"],
                    avg_launch_ms=k[dom]["avg_ms"])
    others = {}
    if not args.no_others:
        for idx in (5, 3, 2, 1):
            if idx == args.workload:
                continue
            r, _ = run_workload(idx, 100, 5, prof=True, timed_events=False)
            others[f"config{idx}"] = r
        # what the headline depends on: the same words against tables of other shapes (a caching
        # allocator's byte-granular blocks; a few 8 GiB regions among the others), and the paper's
        # own archive shape (Section 6.4.1: 512 graphs in about twenty topology groups)
        for key, kind in (("config4_byte_granular_table", "bytes"), ("config4_huge_regions_table", "huge")):
            r, _ = run_workload(4, 10, 2, prof=True, timed_events=False, table_kind=kind,
                                label=f"config 4 words, {kind} table")
            others[key] = r
        edges = [1, 2, 4, 8, 16, 24, 32, 48, 64, 96, 128, 160, 192, 224, 256, 288, 320, 352, 384, 416, 448]
        r, _ = run_workload(2, 50, 5, prof=True, timed_events=False, batch_sizes=list(range(1, 513)),
                            bucket_edges=edges, label="dense decode, 512 graphs in 22 topology groups")
        others["graphs512_templates22"] = r
    out = {
        "metric": "param-blob GB/s (scan+materialize)",
        "value": round(main_res["blob_gbs"], 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(main_res["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64",
        "data": "synthetic",
        "config": {"workload": main_res["workload"], "words": main_res["words"],
                   "allocations": main_res["allocations"], "graphs": main_res["graphs"],
                   "maps": main_res["maps"], "relocs": main_res["relocs"],
                   "step": main_res["step"]},
        "graphs_materialized_per_s": round(main_res["graphs_per_s"], 1),
        "launches_per_step": main_res["launches_per_step"],
        "algorithmic_bytes_per_step": main_res["algorithmic_bytes_per_step"],
        "frac_hbm_peak_step": main_res["frac_hbm_peak_step"],
        "two_call_path": main_res.get("two_call_path"),
        "fused_scan_rebase": main_res.get("fused_scan_rebase"),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": k,
        "other_workloads": others,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
