"""Host-side logic of bench.py and of the profile summariser (no GPU): byte accounting, the provenance
check of the hardware-counter record, the dispatch-plan split, the contract's refusal of several GPUs."""
import json
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench
from paper_2604_16883_amd import binding as B, profile_summary, synth


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""


def test_algorithmic_bytes_and_record_count_by_hand():
    w = synth.WORKLOADS["c1"]                      # B4, 32/8 heads, G = 4
    lens = np.array([32768, 32768, 32768, 32768], np.int32)
    mask = np.ones((4, 8), np.uint8)
    mask[0, 0] = mask[2, 5] = 0                    # two Active Groups of 512 blocks each
    plan = B.sinkrouter_plan(B.make_route_params(4, 32, 8, 32768))
    # per-group shares: 2 groups of 512 blocks share 254 workgroups, 127 each, 5 blocks per share: 103 shares
    # of a group get blocks; 4 heads per group
    assert bench.partial_records(w, lens, mask, plan) == 2 * 4 * 103
    expect = 2 * 32768 * 512 + 2 * 4 * 256 + 2 * 4 * 103 * 520 + 32
    assert bench.algorithmic_bytes(w, lens, mask, plan) == expect
    # more than half as many Active Groups as workgroups: contiguous shares (here B = 40: 160 groups of 512 blocks,
    # 320 blocks per workgroup, so every group's records are the 2 or 3 workgroups its units fall into)
    w2 = synth.Workload("wide", 40, 16, 4, 32768, 0.5)
    plan2 = B.sinkrouter_plan(B.make_route_params(40, 16, 4, 32768))
    units = 512
    c = (160 * units + 255) // 256
    want = sum(4 * (((i + 1) * units - 1) // c - (i * units) // c + 1) for i in range(160))
    assert bench.partial_records(w2, np.full((40,), 32768, np.int32), np.zeros((40, 4), np.uint8), plan2) == want
    # nothing active: only the mask bytes
    assert bench.algorithmic_bytes(w, lens, np.ones((4, 8), np.uint8), plan) == 32
    # fixed chunks: one record per (head, chunk that holds tokens)
    planf = B.sinkrouter_plan(B.make_route_params(4, 32, 8, 32768, num_splits=8))
    lens2 = np.array([32768, 5000, 0, 1], np.int32)
    m2 = np.zeros((4, 8), np.uint8)
    assert planf.chunk_tokens == 4096
    assert bench.partial_records(w, lens2, m2, planf) == 8 * 4 * (8 + 2 + 0 + 1)


def test_counter_record_is_checked_against_the_kernel_sources(tmp_path, monkeypatch):
    sha = bench.kernel_source_sha()
    assert len(sha) == 16 and sha == bench.kernel_source_sha()
    rec = {"c3": {"routed_tau0.55": {"fetch_bytes": 100, "write_bytes": 5, "kernel_source_sha": sha}},
           "c1": {"routed_tau0.55": {"fetch_bytes": 100, "write_bytes": 5, "kernel_source_sha": "0" * 16}}}
    path = tmp_path / "traffic.json"
    path.write_text(json.dumps(rec))
    monkeypatch.setattr(bench, "TRAFFIC_JSON", str(path))
    r, why = bench.measured_traffic("c3", "routed_tau0.55")
    assert r["fetch_bytes"] == 100 and "traffic.json" in why
    r, why = bench.measured_traffic("c1", "routed_tau0.55")
    assert r is None and "other kernel sources" in why
    r, why = bench.measured_traffic("c2", "routed_tau0.55")
    assert r is None and "no counter record" in why
    monkeypatch.setattr(bench, "TRAFFIC_JSON", str(tmp_path / "missing.json"))
    assert bench.measured_traffic("c3", "routed_tau0.55")[0] is None


def test_committed_counter_record_covers_every_workload():
    rec = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
    assert sorted(rec) == ["c0", "c1", "c2", "c3", "c4"]
    for wl, modes in rec.items():
        assert {"routed_tau0.55", "dense"} <= set(modes)
        for mode, r in modes.items():
            ratio = (r["fetch_bytes"] + r["write_bytes"]) / r["algorithmic_bytes"]
            # no wasted re-reads: within 1 % at full size (the 4K-context workload has 0.3 MB of fixed reads on 2 MB)
            assert 0.99 < ratio < (1.01 if wl != "c0" else 1.2), (wl, mode, ratio)
            assert os.path.exists(os.path.join(ROOT, "profiles", "sr_partial_balanced_kernel_%s.md" % wl))


def test_dispatches_are_split_by_the_plan():
    plan = [["a", 3], ["b", 2]]
    assert profile_summary.split_by_plan([1, 2, 3, 4, 5], plan) == {"a": [1, 2, 3], "b": [4, 5]}
    with pytest.raises(SystemExit):
        profile_summary.split_by_plan([1, 2, 3, 4], plan)
    # a third entry says how many of a mode's launches come before its first timed step; without it, the warm-up count
    assert profile_summary.split_by_plan([1, 2, 3, 4, 5], [["a", 3, 2], ["b", 2, 1]]) == {"a": [1, 2, 3], "b": [4, 5]}
    assert profile_summary.leading([["a", 3, 2], ["b", 2]], 1) == {"a": 2, "b": 1}
    assert profile_summary.short("void (anonymous namespace)::sr_partial_balanced_kernel<true, false>(PartialArgs)") == "sr_partial"
    assert profile_summary.short("at::native::vectorized_elementwise_kernel") is None


def test_result_tables_render():
    mode = {"skip_ratio": 0.75, "algorithmic_bytes": 5.0e8, "partial_us": 80.0, "partial_GBps": 6250.0, "partial_frac_of_peak": 0.78,
            "us_per_step": 88.0, "step_GBps": 5700.0, "step_frac_of_peak": 0.71, "combine_us": 4.0}
    paged = dict(mode, partial_us=None, partial_GBps=None, partial_frac_of_peak=None, combine_us=None)
    line = {"steps": 5, "warmup": 1, "seeds": [dict(mode, seed=3000)],
            "detail": {"c3": {"routed_tau0.55": mode, "dense": mode, "routed_tau0.7": mode, "routed_vs_dense_speedup": 3.5},
                       "c1_paged": {"routed_tau0.55": paged, "dense": paged, "routed_vs_dense_speedup": 1.5}},
            "roofline": {"stream_read_probe_GBps": 6700.0, "traffic": None, "traffic_ratio": None, "traffic_source": "none"},
            "cpu_baseline": None}
    md = bench.results_markdown(line)
    assert "| c3 | 0.750 | 500.0 MB | 80.0 | 6250 | 78.0 % | 88.0 |" in md and "n/a" in md and "| 3000 |" in md


def test_profile_summary_end_to_end_on_synthetic_rocprof_output(tmp_path, monkeypatch):
    """The summariser on a hand-made set of rocprofv3 csv files: dispatches attributed to modes by the plan, counter
    units scaled by the copy kernel, warm-up dispatches left out, summary and counter record written."""
    base = tmp_path / "prof_cX"
    for d in ("trace", "fetch", "write"):
        (base / d).mkdir(parents=True)
    plan = [["routed_tau0.55", 3], ["dense", 2]]
    line = {"metric": "m", "steps": 1, "warmup": 1,
            "detail": {"cX": {"description": "test shape", "dispatch_plan": plan,
                              "routed_tau0.55": {"skip_ratio": 0.5, "algorithmic_bytes": 2048000},
                              "dense": {"skip_ratio": 0.0, "algorithmic_bytes": 4096000}}}}
    (base / "trace.log").write_text("noise\n" + json.dumps(line) + "\n")
    part, comb = "void sr_partial_balanced_kernel<true, false>(PartialArgs)", "void sr_combine_kernel<16>(CombineArgs)"
    rows, t = [], 1000
    durs = [9000, 2000, 2200, 4000, 4400]                       # ns; the first of each mode is warm-up
    for d in durs:
        rows.append((part, t, t + d)); t += d + 1500
        rows.append((comb, t, t + 3000)); t += 3000 + 1200
    with open(base / "trace" / "t_kernel_trace.csv", "w") as f:
        f.write("Kernel_Name,Start_Timestamp,End_Timestamp\n")
        for n, a, b in rows:
            f.write('"%s",%d,%d\n' % (n, a, b))
    with open(base / "trace" / "t_kernel_stats.csv", "w") as f:
        f.write("Name,Calls,AverageNs,MinNs,MaxNs\n")
        f.write('"%s",5,4320,2000,9000\n"%s",5,3000,3000,3000\n' % (part, comb))
    for d, name, copy_units, unit in (("fetch", "f", 524288, 2048), ("write", "w", 1048576, 1024)):
        with open(base / d / (name + "_counter_collection.csv"), "w") as f:
            f.write("Kernel_Name,Counter_Value\n")
            f.write('"sr_copy_probe_kernel(uint4*, uint4 const*, unsigned long)",%d\n' % copy_units)
            for i, _ in enumerate(durs):
                bytes_ = (2048000 if i < 3 else 4096000) if d == "fetch" else 10240
                f.write('"%s",%d\n"%s",%d\n' % (part, bytes_ // unit, comb, 1))
    # an optional further pass with two instruction counters, two hardware instances per dispatch (summed)
    (base / "insts").mkdir()
    (base / "insts.log").write_text(json.dumps(line) + "\n")
    with open(base / "insts" / "p_counter_collection.csv", "w") as f:
        f.write("Dispatch_Id,Kernel_Name,Counter_Name,Counter_Value\n")
        for i, _ in enumerate(durs):
            blocks = 62 if i < 3 else 125
            for name, per_block in (("SQ_INSTS_MFMA", 48), ("SQ_INSTS_VALU", 400), ("SQ_INSTS_VMEM_RD", 32)):
                for inst in range(2):
                    f.write('%d,"%s",%s,%d\n' % (2 * i + 1, part, name, blocks * per_block // 2))
            f.write('%d,"%s",SQ_INSTS_MFMA,%d\n' % (2 * i + 2, comb, 0))
    monkeypatch.setattr(profile_summary, "ROOT", str(tmp_path))
    profile_summary.main(["x", str(base), "cX"])
    rec = json.load(open(tmp_path / "profiles" / "traffic.json"))["cX"]
    r = rec["routed_tau0.55"]
    assert r["fetch_bytes"] == 2048000 and r["write_bytes"] == 10240 and r["trace_us_mean"] == 2.1 and r["trace_us_min"] == 2.0
    assert rec["dense"]["fetch_bytes"] == 4096000 and rec["dense"]["trace_us_mean"] == 4.4
    assert r["kernel_source_sha"] == bench.kernel_source_sha() and r["fetch_unit_bytes"] == 2048.0
    md = open(tmp_path / "profiles" / "sr_partial_balanced_kernel_cX.md").read()
    assert "| routed_tau0.55 | 0.500 | 2.1 / 2.0 | 2.05 | 2.05 | 0.01 | 1.0050 |" in md and "rocprofv3 --pmc FETCH_SIZE" in md
    assert "| SQ_INSTS_MFMA | 2976 | 6000 |" in md and "(dense): 48 MFMA, 400 VALU and 32.0 vector-memory" in md
    assert "| 3.0 | 1.50 |" in md                                 # merge kernel duration and the gap behind the partial kernel
