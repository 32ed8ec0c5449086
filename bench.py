#!/usr/bin/env python3
"""Benchmark of the routed decode-attention hot path on one MI355X.

A "step" is one decode step of one attention layer: routing probe, Split-K partial
attention over the Active Groups, log-sum-exp merge, on a seeded synthetic KV cache that
is resident in HBM before the timed region.  The headline workload is the 512K-context
Llama-3.1-70B-shaped layer (c3); the other four workloads (c0, c1 = 128K tokens, c2, c4),
c3 at the paper's ~60 % skip ratio, a ragged 128K-class batch (contiguous and paged) and the
in-house dense Split-K run on the same inputs are reported in the same JSON line.

Prints ONE JSON line: metric / value (microseconds per step, lower is better), the
roofline record of the dominant kernel (Split-K partial: algorithmic HBM bytes over its
own duration, from HIP events attached to the launch, against 8 TB/s) and the CPU oracle
timed on the same inputs.

Other modes: --lean (one workload, nothing else: the run the profiler wraps), --timeline
(per-phase accounting from the measurement build), --markdown PATH (the result tables).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E bandwidth
D = 128
TAU = 0.55                # the paper's operating threshold (Appendix A)
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")
# sources that decide what the partial kernel reads and writes: a counter record is valid for these only
KERNEL_SOURCES = ["sr_config.h", "sr_common.h", "sr_route.h", "sr_partial.h"]
RAGGED_LENS = [32768, 20011, 4097, 65]      # c1-shaped batch with one long and several short sequences
PRECONDITION_S = 0.1      # seconds of untimed calls in front of every timed mode (see precondition)
CONTEXT_SWEEP = [8192, 16384, 32768, 65536, 131072, 262144]   # c3-shaped layer at shorter contexts (512K is the headline)


def kernel_source_sha() -> str:
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2604_16883_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, mode: str):
    """HBM bytes per launch of the partial kernel from the committed rocprofv3 counter record
    (profiles/traffic.json, written by paper_2604_16883_amd.profile_summary), or (None, reason)
    when there is none for this workload and mode or it was taken on other kernel sources."""
    try:
        rec = json.load(open(TRAFFIC_JSON))
    except (OSError, ValueError):
        return None, "no profiles/traffic.json"
    r = rec.get(workload, {}).get(mode)
    if r is None:
        return None, "no counter record for %s %s" % (workload, mode)
    if r.get("kernel_source_sha") != kernel_source_sha():
        return None, "counter record of %s %s was taken on other kernel sources (%s, now %s)" % (
            workload, mode, r.get("kernel_source_sha"), kernel_source_sha())
    return r, "profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by the copy kernel of the same run"


def per_group_shares(units, P):
    """The balanced schedule's choice, mirrored from the kernel: every Active Group gets workgroups of its own if at most
    half as many groups are active as there are workgroups and the shares then occupy at least three quarters of them."""
    U, A = sum(units), sum(1 for u in units if u)
    if not U or 2 * A > P:
        return False
    return 4 * sum((u * (P - A) + U - 1) // U for u in units if u) >= 3 * P


def partial_records(w, seq_lens, mask, plan):
    """Number of (head, workgroup) partial records the Split-K kernel writes for this mask."""
    B, Hq, Hkv = w.batch, w.n_q_heads, w.n_kv_heads
    G = Hq // Hkv
    if plan.schedule == 0:
        return sum(G * ((int(seq_lens[b]) + plan.chunk_tokens - 1) // plan.chunk_tokens)
                   for b in range(B) for g in range(Hkv) if not mask[b, g])
    units = [0 if mask[b, g] else (int(seq_lens[b]) + 63) // 64 for b in range(B) for g in range(Hkv)]
    U, P = sum(units), plan.partial_grid
    A = sum(1 for u in units if u)
    if U == 0:
        return 0
    if per_group_shares(units, P):
        # per-group shares: group i gets ceil(u_i (P - A) / U) workgroups of ceil(u_i / n_i) blocks each
        n = 0
        for u in units:
            if u:
                ni = (u * (P - A) + U - 1) // U
                cb = (u + ni - 1) // ni
                n += G * ((u + cb - 1) // cb)
        return n
    c = (U + P - 1) // P
    n, s0 = 0, 0
    for u in units:
        if u:
            n += G * ((s0 + u - 1) // c - s0 // c + 1)
        s0 += u
    return n


def algorithmic_bytes(w, seq_lens, mask, plan):
    """Bytes the method itself must move in the Split-K partial kernel for this mask:
    K and V rows of every Active Group once (shared by the group's heads), the group's
    queries, the routing bytes, and the partial (m, l, o) records it writes."""
    B, Hq, Hkv = w.batch, w.n_q_heads, w.n_kv_heads
    G = Hq // Hkv
    total = 0
    for b in range(B):
        for g in range(Hkv):
            if not mask[b, g]:
                total += int(seq_lens[b]) * D * 2 * 2       # K + V rows
                total += G * D * 2                          # the group's queries (once)
    total += partial_records(w, seq_lens, mask, plan) * (D + 2) * 4
    total += B * Hkv                                         # skip bytes
    return total


def time_steps(fn, steps, warmup, both=False):
    """`warmup` untimed calls, then exactly `steps` timed calls between two device synchronisations.  The figure is the
    time the device took for them: two events on the launch stream.  One more untimed call follows the first
    synchronisation and the first event is recorded behind it, so that the event's time stamp is taken when that call
    ends, with the first timed call already queued: otherwise the device idles until the host's first launch arrives and
    a short run is charged for it (about 0.5 us per step at 20 steps).  The host clock around the same bracket (over all
    `steps` + 1 calls) also counts the host's wake-up after the last kernel, 15-25 us per bracket: 1 us per step at 20
    steps, 0.04 at 500; with `both` it is returned as well."""
    import torch
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    fn()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    host = (time.perf_counter() - t0) / (steps + 1) * 1e6
    dev = e0.elapsed_time(e1) * 1e3 / steps
    return (dev, host) if both else dev


def precondition(fn, seconds=0.1):
    """Keeps the device busy with the calls about to be timed for `seconds` before their warm-up steps.  After idling
    (the wait in settle(), a process start) the first 8-10 ms of work run up to 6 % slower and the step time keeps
    falling slightly for some 100 ms (512K-context step: 89.2 us in the first 9 ms, 86.8-87.2 us until 80 ms, then
    86.5 us), which 50 warm-up steps of 10-90 us do not cover; a serving device is never idle between decode steps."""
    import torch
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(50):
            fn()
        torch.cuda.synchronize()


def settle():
    """Frees the cached device memory and waits for the device to get over it.  For some hundred milliseconds after
    gigabytes of device memory are released every kernel streams 3-4 % slower (the 128K-token step: 41.7 instead of
    40.2 us for at least 140 ms after an 8 GiB buffer is freed, back to 40.2 us a second later; allocating has no
    such effect), so a workload timed right after its predecessor's buffers were freed would be charged for that."""
    import torch
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    time.sleep(1.5)


def auto_copies(kv_bytes):
    """Distinct K/V copies to rotate through so that a step finds (almost) none of its rows in the 256 MB memory-side
    cache: the rows a routed step touches (as little as a fifth of the cache at a skip ratio of 0.8), summed over the
    rotation, are at least six times the cache.  Measured on the 128K-token batch: 38.8 us per routed step with 3 copies,
    39.1 with 4, 40.4 with 6, 8, 12 and 16.  Short contexts need hundreds of copies (a 4K-token cache is 17 MB); the
    rotation is capped at 512 copies and 32 GB."""
    want = -(-6 * 256e6 // (0.2 * kv_bytes))
    return int(max(3, min(want, 512, 32e9 // kv_bytes)))


class Case:
    """One workload resident in HBM: queries, lengths, `copies` distinct copies of K and V (rotated so that
    no step finds its rows in the last-level cache; 0 = auto_copies), and the anchors a prefill would have cached."""

    def __init__(self, name, copies, seed=None, seq_lens=None, page_tokens=0):
        import torch
        from paper_2604_16883_amd import binding, synth
        w = synth.WORKLOADS[name]
        if seq_lens is not None:
            w = w.scaled(max(seq_lens), batch=len(seq_lens), name="%s ragged" % name)
        if not copies:
            lens = seq_lens if seq_lens is not None else [w.seq_len] * w.batch
            copies = auto_copies(sum(lens) * w.n_kv_heads * D * 2 * 2)
        t0 = time.time()
        sb = synth.generate(w, seed=seed, seq_lens=seq_lens, threads=min(16, os.cpu_count() or 8))
        self.gen_s = time.time() - t0
        self.w, self.sb, self.copies, self.page_tokens = w, sb, copies, page_tokens
        self.B, self.Hq, self.Hkv, self.Lmax = w.batch, w.n_q_heads, w.n_kv_heads, sb.max_seq_len
        self.q = torch.from_numpy(sb.q.view(np.int16)).cuda()
        self.sl = torch.from_numpy(sb.seq_lens).cuda()
        self.layout = self.table = None
        if page_tokens:
            # the same cache scattered into a page pool in a seeded random page order
            kp, tab = synth.to_pages(sb.k, sb.seq_lens, page_tokens, seed=w.base_seed)
            vp, _ = synth.to_pages(sb.v, sb.seq_lens, page_tokens, seed=w.base_seed)
            k0, v0 = torch.from_numpy(kp.view(np.int16)).cuda(), torch.from_numpy(vp.view(np.int16)).cuda()
            self.table = torch.from_numpy(tab).cuda()
            self.layout = binding.make_paged_layout(page_tokens, tab.shape[1], kp.shape[0])
            del kp, vp
        else:
            k0 = torch.from_numpy(sb.k.view(np.int16)).cuda()
            v0 = torch.from_numpy(sb.v.view(np.int16)).cuda()
        # all copies of K in one allocation and all copies of V in another, as the layers of a model's cache would be:
        # hundreds of separate small buffers, freed again, leave the device memory fragmented for whatever is allocated
        # next (measured: the 128K-token batch then runs 3-4 % slower for the rest of the process)
        k_all = torch.empty((copies,) + tuple(k0.shape), dtype=k0.dtype, device="cuda")
        v_all = torch.empty((copies,) + tuple(v0.shape), dtype=v0.dtype, device="cuda")
        k_all[:] = k0
        v_all[:] = v0
        del k0, v0
        self.ks = [k_all[i] for i in range(copies)]
        self.vs = [v_all[i] for i in range(copies)]
        self.out = torch.empty((self.B, self.Hq, D), dtype=torch.int16, device="cuda")
        self.mask = torch.empty((self.B, self.Hkv), dtype=torch.uint8, device="cuda")
        # prefill-side anchor caching (Section 4.1): K_0 and its norm are extracted once per sequence, by the
        # library's own kernel, outside the timed region; the contents are the same for every copy
        self.k0 = torch.from_numpy(np.ascontiguousarray(sb.k[:, :, 0]).view(np.int16)).cuda()
        self.k0_norm = torch.empty((self.B, self.Hkv), dtype=torch.float32, device="cuda")
        binding.sinkrouter_extract_anchor(self.k0, binding.make_route_params(self.B, self.Hq, self.Hkv, 1), None, self.k0_norm)
        torch.cuda.synchronize()

    def params(self, routing, tau, cached_anchors, num_splits=0):
        import torch
        from paper_2604_16883_amd import binding
        p = binding.make_route_params(self.B, self.Hq, self.Hkv, self.Lmax, routing_enabled=routing, tau_coef=(0, 0, 0, tau),
                                      num_splits=num_splits, k0=self.k0 if cached_anchors else None,
                                      k0_norm=self.k0_norm if cached_anchors else None)
        plan = binding.sinkrouter_plan(p)
        ws = torch.empty((plan.workspace_bytes,), dtype=torch.uint8, device="cuda")
        p.workspace, p.workspace_bytes = ws.data_ptr(), plan.workspace_bytes
        return p, plan, ws

    def call(self, p, i, profiled=False):
        from paper_2604_16883_amd import binding
        i %= self.copies
        if self.layout is not None:
            return binding.sinkrouter_decode_paged(self.q, self.ks[i], self.vs[i], self.table, self.sl, p, self.layout, self.out, self.mask)
        if profiled:
            return binding.sinkrouter_decode_profiled(self.q, self.ks[i], self.vs[i], self.sl, p, self.out, self.mask)
        return binding.sinkrouter_decode(self.q, self.ks[i], self.vs[i], self.sl, p, self.out, self.mask)

    def time_mode(self, steps, warmup, routing=True, tau=TAU, cached_anchors=True, num_splits=0, use_graph=False):
        """Times one configuration: wall clock over `steps` asynchronous calls, the spread of the step time, and
        per-kernel durations from HIP events attached to the launches (separate, synchronous *_profiled calls)."""
        import torch
        p, plan, ws = self.params(routing, tau, cached_anchors, num_splits)
        it = [0]

        def step():
            self.call(p, it[0])
            it[0] += 1

        launches = [0]

        def counted():
            step()
            launches[0] += 1

        precondition(counted, PRECONDITION_S)
        leading = launches[0] + warmup + 1          # launches of this mode before the first timed one
        us, host_us = time_steps(step, steps, warmup, both=True)
        launches = leading + steps
        graph_us = None
        if use_graph:
            # the same steps replayed from one HIP graph (one decode call per K/V copy)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            it[0] = 0
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(self.copies):
                    step()
            reps = max(1, steps // self.copies)
            graph_us = time_steps(g.replay, reps, max(1, warmup // self.copies)) / self.copies
            launches += 1 + self.copies * (reps + 1 + max(1, warmup // self.copies))
        # spread of the step time: one event between consecutive asynchronous steps, same rotation
        n_marks, n_prof = min(max(steps, 50), 200), 100      # not fewer when a run times only a few steps
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_marks + 1)]
        it[0] = 0
        for s in range(n_marks):
            marks[s].record()
            step()
        marks[n_marks].record()
        torch.cuda.synchronize()
        step_us = np.array([marks[s].elapsed_time(marks[s + 1]) * 1e3 for s in range(n_marks)])
        launches += n_marks
        st = np.zeros((n_prof, 4))
        if self.layout is None:
            for s in range(n_prof):
                st[s] = self.call(p, s, profiled=True)
            launches += n_prof
        torch.cuda.synchronize()
        m = self.mask.cpu().numpy()
        ab = algorithmic_bytes(self.w, self.sb.seq_lens, m, plan)
        # no per-kernel events for the paged entry point: whole step only
        partial_us = float(np.mean(st[:, 1])) if self.layout is None else None
        return {
            "us_per_step": round(us, 2), "us_per_step_host_clock": round(host_us, 2),
            "us_per_step_graph_replay": None if graph_us is None else round(graph_us, 2),
            "step_us_p10_p50_p90": [round(float(x), 2) for x in np.percentile(step_us, [10, 50, 90])],
            "probe_us": round(float(np.mean(st[:, 0])), 2),
            "partial_us": None if partial_us is None else round(partial_us, 2),
            "partial_us_p10_p50_p90": [round(float(x), 2) for x in np.percentile(st[:, 1], [10, 50, 90])],
            "combine_us": None if partial_us is None else round(float(np.mean(st[:, 2])), 2),
            "skip_ratio": round(float(m.mean()), 4),
            "active_groups": int((1 - m).sum()),
            "algorithmic_bytes": int(ab),
            "partial_GBps": None if partial_us is None else round(ab / partial_us / 1e3, 1),
            "partial_frac_of_peak": None if partial_us is None else round(ab / partial_us / 1e3 / HBM_PEAK_GBS, 4),
            "step_GBps": round(ab / us / 1e3, 1),
            "step_frac_of_peak": round(ab / us / 1e3 / HBM_PEAK_GBS, 4),
            "anchors": "prefill-cached k0 and k0_norm" if (cached_anchors and routing) else ("row 0 of the cache" if routing else "unused"),
            "schedule": "balanced" if plan.schedule else "fixed", "page_tokens": self.page_tokens,
            "partial_grid": int(plan.partial_grid), "partial_records": partial_records(self.w, self.sb.seq_lens, m, plan),
            "partial_kernel_launches": launches, "leading_untimed_launches": leading,
        }


def run_workload(name, steps, warmup, copies, verbose, num_splits=0, page_tokens=0, use_graph=False, seed=None, seq_lens=None,
                 taus=True, prefill_anchors=True):
    """All modes of one workload.  'routed_tau0.55' does all of the step's work inside the step: K_0 is read from
    row 0 of the key cache and its norm recomputed; 'routed_tau0.55_prefill_anchors' routes on the K_0 tensor and norm
    a prefill would have cached (Section 4.1)."""
    case = Case(name, copies, seed=seed, seq_lens=seq_lens, page_tokens=page_tokens)
    res = {"workload": name, "description": case.w.description if seq_lens is None else
           "%s-shaped batch with ragged lengths %s" % (name, list(seq_lens)), "seed": case.sb.seed,
           "gen_s": round(case.gen_s, 2), "copies": case.copies}
    kw = dict(num_splits=num_splits, use_graph=use_graph)
    modes = [("routed_tau0.55", dict(routing=True, tau=TAU, cached_anchors=False))]
    if prefill_anchors:
        modes.append(("routed_tau0.55_prefill_anchors", dict(routing=True, tau=TAU, cached_anchors=True)))
    if taus:
        modes += [("routed_tau%.3f" % t, dict(routing=True, tau=t, cached_anchors=False)) for t in case.sb.taus[1:]]
    modes.append(("dense", dict(routing=False, tau=TAU, cached_anchors=False)))
    plan_order = []
    for label, m in modes:
        r = case.time_mode(steps, warmup, **m, **kw)
        res[label] = r
        plan_order.append([label, r["partial_kernel_launches"], r["leading_untimed_launches"]])
        if verbose:
            print(name, label, r, file=sys.stderr, flush=True)
    res["dispatch_plan"] = plan_order
    res["routed_vs_dense_speedup"] = round(res["dense"]["us_per_step"] / res["routed_tau0.55"]["us_per_step"], 3)
    return res, case


def headline(r):
    """The figures of one workload that go into the `also` record."""
    rt, dn = r["routed_tau0.55"], r["dense"]
    return {"workload": r["description"], "us_per_step": rt["us_per_step"], "dense_us_per_step": dn["us_per_step"],
            "skip_ratio": rt["skip_ratio"], "algorithmic_bytes": rt["algorithmic_bytes"],
            "partial_kernel_us": rt["partial_us"], "partial_kernel_GBps": rt["partial_GBps"],
            "partial_kernel_frac_of_peak": rt["partial_frac_of_peak"],
            "step_GBps": rt["step_GBps"], "step_frac_of_peak": rt["step_frac_of_peak"],
            "dense_partial_kernel_frac_of_peak": dn["partial_frac_of_peak"], "dense_step_frac_of_peak": dn["step_frac_of_peak"],
            "routed_vs_dense_speedup": r["routed_vs_dense_speedup"]}


def timeline_report(name, tau, steps, copies, anchors_cached):
    """Per-phase accounting of one routed step from the measurement build of the library (every workgroup
    leaves wall-clock stamps, 100 MHz counter): medians over workgroups and steps, microseconds after the
    first workgroup of the partial kernel entered."""
    import torch
    from paper_2604_16883_amd import binding
    nbytes = binding.sinkrouter_timeline_bytes()
    if nbytes == 0:
        raise SystemExit("bench.py --timeline needs the measurement build: python -m paper_2604_16883_amd.build --timeline")
    case = Case(name, copies)
    w, sb = case.w, case.sb
    B, Hq, Hkv = case.B, case.Hq, case.Hkv
    routing = tau < 2.0
    p, plan, ws = case.params(routing, tau, anchors_cached and routing)
    ws.zero_()
    stamps = ws[plan.workspace_bytes - nbytes:]
    grid = plan.partial_grid
    rows_p, rows_m, ev_us = [], [], []
    for s in range(steps + 5):
        stamps.zero_()
        torch.cuda.synchronize()
        case.call(p, s)                                   # the plain call: kernels back to back
        torch.cuda.synchronize()
        if s < 5:
            continue
        t = stamps.cpu().numpy().view(np.int64).astype(np.float64) / 100.0       # microseconds
        if s % 4 == 0:
            ev_us.append(case.call(p, s + 1, profiled=True))
        tp = t[:grid * 8].reshape(grid, 8)
        tm = t[grid * 8:].reshape(-1, 4)
        # a head's merge may be split over several workgroups (column parts): entry = first of them, the rest = last
        parts = max(int((tm[:, 0] > 0).sum()) // (B * Hq), 1)
        tm = tm[:B * Hq * parts].reshape(B * Hq, parts, 4)
        tm = np.concatenate([tm[..., :1].min(axis=1), tm[..., 1:].max(axis=1)], axis=1)
        t0 = tp[:, 0].min()
        rows_p.append(tp - t0)
        rows_m.append(tm - t0)
    m = case.mask.cpu().numpy()
    tp = np.stack(rows_p)                  # [steps, grid, 8]
    tm = np.stack(rows_m)                  # [steps, heads, 4]
    busy = tp[..., 5] > 0                  # workgroups that streamed something
    units = [0 if m[b, g] else (int(sb.seq_lens[b]) + 63) // 64 for b in range(B) for g in range(Hkv)]
    U, A = sum(units), sum(1 for u in units if u)
    if per_group_shares(units, grid):           # the largest share of any group
        c = max((u + ((u * (grid - A) + U - 1) // U) - 1) // ((u * (grid - A) + U - 1) // U) for u in units if u)
    else:
        c = (U + grid - 1) // grid
    steps_wave0 = (c + 3) // 4

    def med(x):
        return round(float(np.median(x)), 2)

    def sel(j):
        return tp[..., j][busy]

    merged = np.repeat(1 - m.reshape(-1), Hq // Hkv).astype(bool)          # heads that have records
    ab = algorithmic_bytes(w, sb.seq_lens, m, plan)
    ev = np.array(ev_us)
    first_issue, last_exit = med(sel(3)), med(tp[..., 7].max(axis=1))
    return {
        "workload": name, "tau": tau, "skip_ratio": round(float(m.mean()), 4), "anchors_cached": bool(anchors_cached and routing),
        "blocks_per_workgroup": c, "block_steps_of_wavefront_0": steps_wave0, "busy_workgroups": int(busy[0].sum()),
        "algorithmic_bytes": int(ab),
        "stream_GBps_first_issue_to_last_exit": round(ab / max(last_exit - first_issue, 1e-9) / 1e3, 1),
        "partial": {
            "entry_spread_p50_max": [med(sel(0)), round(float(np.median(tp[..., 0].max(axis=1))), 2)],
            "probe_end": med(sel(1)), "barrier_passed": med(sel(2)), "schedule_end": first_issue,
            "first_block_done": med(sel(4)), "stream_end": med(sel(5)), "records_written": med(sel(6)),
            "exit_p50": med(sel(7)), "exit_last": last_exit,
            # the same phases as durations inside one workgroup (its own entry = 0)
            "own_probe": med(sel(1) - sel(0)), "own_schedule": med(sel(3) - sel(2)), "own_first_block": med(sel(4) - sel(3)),
            "own_stream_rest": med(sel(5) - sel(4)), "own_records": med(sel(6) - sel(5)),
        },
        "gap_partial_exit_to_merge_entry": med(tm[..., 0].min(axis=1) - tp[..., 7].max(axis=1)),
        "merge": {
            "entry_first": med(tm[..., 0].min(axis=1)), "entry_last": med(tm[..., 0].max(axis=1)),
            "records_loaded": med(tm[:, merged, 1]) if merged.any() else None,
            "merged": med(tm[:, merged, 2]) if merged.any() else None,
            "exit_last": med(tm[..., 3].max(axis=1)),
            "own_load": med(tm[:, merged, 1] - tm[:, merged, 0]) if merged.any() else None,
            "own_barrier": med(tm[:, merged, 2] - tm[:, merged, 1]) if merged.any() else None,
            "own_finish": med(tm[:, merged, 3] - tm[:, merged, 2]) if merged.any() else None,
        },
        "events_us": {"partial_kernel": med(ev[:, 1]), "merge_kernel": med(ev[:, 2])},
    }


def timeline_markdown(rep, read_gbs):
    """The accounting as a markdown table, with the time the bytes take at the streaming-read rate beside it."""
    p, mg = rep["partial"], rep["merge"]
    ideal = rep["algorithmic_bytes"] / read_gbs / 1e3
    rows = [
        ("partial kernel: last workgroup enters", p["entry_spread_p50_max"][1]),
        ("probe done (cosines of all groups in LDS)", p["probe_end"]),
        ("barrier behind the probe passed", p["barrier_passed"]),
        ("schedule built, first K/V loads issued", p["schedule_end"]),
        ("first 64-token block step done", p["first_block_done"]),
        ("last block step done (stream end)", p["stream_end"]),
        ("partial records written", p["records_written"]),
        ("workgroup exit, median / last", "%s / %s" % (p["exit_p50"], p["exit_last"])),
        ("merge kernel: first / last workgroup enters", "%s / %s" % (mg["entry_first"], mg["entry_last"])),
        ("merge: records loaded", mg["records_loaded"]),
        ("merge: merged through LDS", mg["merged"]),
        ("merge: last workgroup exits", mg["exit_last"]),
    ]
    label = "dense (routing off)" if rep["tau"] >= 2.0 else "tau %s, skip ratio %s, anchors %s" % (
        rep["tau"], rep["skip_ratio"], "prefill-cached" if rep["anchors_cached"] else "read from row 0 of the cache")
    out = ["### %s, %s" % (rep["workload"], label), "",
           "| point in the step (medians over workgroups and steps) | us after the first workgroup entered |", "|---|---|"]
    out += ["| %s | %s |" % r for r in rows]
    out += ["",
            "%d blocks per workgroup, %d block steps for wavefront 0; %d of 256 workgroups stream."
            % (rep["blocks_per_workgroup"], rep["block_steps_of_wavefront_0"], rep["busy_workgroups"]),
            "Inside one workgroup of the partial kernel (medians): probe %s us, schedule %s us, first block step %s us, the other "
            "block steps %s us, merge of its 4 wavefronts and record write %s us.  Inside one merge workgroup: records loaded after %s us, "
            "barrier passed %s us later, output written and exit %s us later."
            % (p["own_probe"], p["own_schedule"], p["own_first_block"], p["own_stream_rest"], p["own_records"],
               mg["own_load"], mg["own_barrier"], mg["own_finish"]),
            "Gap between the last partial workgroup's exit and the first merge workgroup's entry: %s us."
            % rep["gap_partial_exit_to_merge_entry"],
            "Algorithmic bytes %.1f MB: %.1f us at the streaming-read rate measured in the same run (%.0f GB/s), %.1f us at 8 TB/s; "
            "from the first K/V load to the last exit the kernel moves them at %.0f GB/s."
            % (rep["algorithmic_bytes"] / 1e6, ideal, read_gbs, rep["algorithmic_bytes"] / 8e6, rep["stream_GBps_first_issue_to_last_exit"]),
            "HIP events attached to the launches, same inputs: partial kernel %s us, merge kernel %s us (an empty kernel reads 3.9 us by "
            "these events: they include dispatch and completion handling)." % (rep["events_us"]["partial_kernel"], rep["events_us"]["merge_kernel"]), ""]
    return "\n".join(out)


def _f(x, fmt="%.1f", scale=1.0):
    return "n/a" if x is None else fmt % (x * scale)


def results_markdown(line):
    """The result tables of the design notes, generated from one benchmark line."""
    det = line["detail"]
    out = ["<!-- generated by: python bench.py --markdown <this file>; do not edit -->", "",
           "Benchmark results on one MI355X, %d timed steps after %d warm-up steps per mode (no per-kernel events exist for the paged entry point: n/a)." % (line["steps"], line["warmup"]), "",
           "Partial kernel (events attached to the launch) and whole step (wall clock), routed at tau = 0.55 (K_0 read from the cache, norm recomputed):", "",
           "| workload | skip | bytes | partial kernel us | GB/s | of 8 TB/s | step us | step GB/s | of 8 TB/s | dense step us | speed-up |",
           "|---|---|---|---|---|---|---|---|---|---|---|"]
    for name in sorted(det):
        r = det[name]
        rt, dn = r["routed_tau0.55"], r["dense"]
        out.append("| %s | %.3f | %.1f MB | %s | %s | %s %% | %.1f | %.0f | %.1f %% | %.1f | %.2fx |" % (
            name, rt["skip_ratio"], rt["algorithmic_bytes"] / 1e6, _f(rt["partial_us"]), _f(rt["partial_GBps"], "%.0f"),
            _f(rt["partial_frac_of_peak"], "%.1f", 100), rt["us_per_step"], rt["step_GBps"], 100 * rt["step_frac_of_peak"], dn["us_per_step"], r["routed_vs_dense_speedup"]))
    out += ["", "Dense Split-K (routing off) on the same inputs:", "",
            "| workload | bytes | partial kernel us | of 8 TB/s | step us | of 8 TB/s |", "|---|---|---|---|---|---|"]
    for name in sorted(det):
        dn = det[name]["dense"]
        out.append("| %s | %.1f MB | %s | %s %% | %.1f | %.1f %% |" % (
            name, dn["algorithmic_bytes"] / 1e6, _f(dn["partial_us"]), _f(dn["partial_frac_of_peak"], "%.1f", 100), dn["us_per_step"],
            100 * dn["step_frac_of_peak"]))
    out += ["", "Other modes (us per step):", "", "| workload | mode | skip | step us | partial kernel us | merge kernel us |", "|---|---|---|---|---|---|"]
    for name in sorted(det):
        for mode, r in det[name].items():
            if isinstance(r, dict) and "us_per_step" in r and mode not in ("routed_tau0.55", "dense"):
                out.append("| %s | %s | %.3f | %.1f | %s | %s |" % (name, mode, r["skip_ratio"], r["us_per_step"], _f(r["partial_us"]), _f(r["combine_us"])))
    if line.get("seeds"):
        out += ["", "c3 over repetition seeds (routed, tau = 0.55):", "", "| seed | skip | bytes | step us | step of 8 TB/s | partial kernel of 8 TB/s |",
                "|---|---|---|---|---|---|"]
        for s in line["seeds"]:
            out.append("| %d | %.3f | %.1f MB | %.1f | %.1f %% | %.1f %% |" % (s["seed"], s["skip_ratio"], s["algorithmic_bytes"] / 1e6, s["us_per_step"],
                                                                       100 * s["step_frac_of_peak"], 100 * s["partial_frac_of_peak"]))
    pts = (line.get("context_sweep") or {}).get("points") or []
    if pts:
        main = det.get("c3")
        out += ["", "Step time against context length, c3-shaped layer (B1, 64 query / 8 KV heads), routed at tau = 0.55 and dense on identical "
                "inputs (Section 5.3 of the paper reports small gains below 64K tokens, growing with the context):", "",
                "| context | skip | K/V copies rotated | routed step us | of 8 TB/s | dense step us | of 8 TB/s | speed-up |", "|---|---|---|---|---|---|---|---|"]
        for s in pts:
            out.append("| %d | %.3f | %d | %.1f | %.1f %% | %.1f | %.1f %% | %.2fx |" % (
                s["context"], s["skip_ratio"], s["copies"], s["us_per_step"], 100 * s["step_frac_of_peak"], s["dense_us_per_step"],
                100 * s["dense_step_frac_of_peak"], s["routed_vs_dense_speedup"]))
        if main:
            rt, dn = main["routed_tau0.55"], main["dense"]
            out.append("| 524288 | %.3f | %d | %.1f | %.1f %% | %.1f | %.1f %% | %.2fx |" % (
                rt["skip_ratio"], main["copies"], rt["us_per_step"], 100 * rt["step_frac_of_peak"], dn["us_per_step"],
                100 * dn["step_frac_of_peak"], main["routed_vs_dense_speedup"]))
    rf, cpu = line["roofline"], line["cpu_baseline"]
    out += ["", "Streaming-read probe of the same run: %.0f GB/s.  HBM traffic of the partial kernel from hardware counters: %s "
            "(%s)." % (rf["stream_read_probe_GBps"], "%.1f MB = %.4f x the algorithmic bytes" % (rf["traffic"] / 1e6, rf["traffic_ratio"])
                       if rf["traffic"] else "none", rf["traffic_source"])]
    if cpu:
        out.append("CPU oracle on the same inputs: %.0f us per routed step on %d host threads (%s)." % (cpu["value"], cpu["cores"], cpu["sample"]))
    return "\n".join(out) + "\n"


BATCH_SWEEP = [(8, 8192, False), (16, 16384, False), (32, 8192, False), (64, 8192, False), (64, 4096, False), (128, 4096, False),
               (32, 8192, True), (64, 8192, True)]


def batch_sweep_markdown(steps, warmup):
    """Large batches of short contexts (the serving regime; none of the paper's workloads): the 8B-shaped layer (32 query /
    8 KV heads) with B sequences of L tokens, or of seeded ragged lengths in [0.15 L, L]; routed at tau = 0.55 and dense."""
    out = ["Large batches on the 8B-shaped layer (32 query / 8 KV heads), routed at tau = 0.55 and dense (routing off); fraction of 8 TB/s "
           "on the bytes read; `python bench.py --batch-sweep`:", "",
           "| sequences | context | lengths | groups | active | probe | routed step us | of 8 TB/s | dense step us | of 8 TB/s | speed-up |",
           "|---|---|---|---|---|---|---|---|---|---|---|"]
    for B, L, ragged in BATCH_SWEEP:
        rng = np.random.default_rng(B * 1000 + L)
        lens = [int(L * f) for f in rng.uniform(0.15, 1.0, B)] if ragged else [L] * B
        lens[0] = L
        case = Case("c1", 0, seq_lens=lens)
        r = case.time_mode(steps, warmup, routing=True, tau=TAU, cached_anchors=False)
        d = case.time_mode(steps, warmup, routing=False, tau=TAU, cached_anchors=False)
        out.append("| %d | %d | %s | %d | %d | %s | %.1f | %.1f %% | %.1f | %.1f %% | %.2fx |" % (
            B, L, "ragged" if ragged else "equal", B * 8, r["active_groups"], "separate launch" if r["probe_us"] else "fused",
            r["us_per_step"], 100 * r["step_frac_of_peak"], d["us_per_step"], 100 * d["step_frac_of_peak"], d["us_per_step"] / r["us_per_step"]))
        del case
        settle()
    return "\n".join(out)


def hbm_calibration(nbytes=2 << 30, reps=10):
    """Achieved streaming-read bandwidth of a plain 128-bit read kernel (context for the roofline)."""
    import torch
    from paper_2604_16883_amd import binding
    buf = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
    buf.random_(0, 255)
    sink = torch.zeros((4096,), dtype=torch.uint8, device="cuda")
    binding.sinkrouter_hbm_read_probe(buf, nbytes, sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        binding.sinkrouter_hbm_read_probe(buf, nbytes, sink)
    e1.record()
    torch.cuda.synchronize()
    read_gbs = nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    # one plain copy of known size: the reference dispatch for scaling hardware byte counters
    dst = torch.empty((nbytes // 2,), dtype=torch.uint8, device="cuda")
    binding.sinkrouter_hbm_copy_probe(dst, buf, nbytes // 2)
    torch.cuda.synchronize()
    return read_gbs


def cpu_baseline(sb, budget_s=20.0):
    """The fp64 oracle, as it stands, on the same inputs and the same routed step (tau = 0.55) that
    `value` times, on the machine's host cores; repeated up to three times within the time budget."""
    import oracle
    times = []
    t_all = time.perf_counter()
    for _ in range(3):
        t0 = time.perf_counter()
        oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=(0, 0, 0, TAU), diagnostics=False)
        times.append(time.perf_counter() - t0)
        if time.perf_counter() - t_all > budget_s:
            break
    t0 = time.perf_counter()
    oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, routing_enabled=False, diagnostics=False)
    dense_s = time.perf_counter() - t0
    return {"value": round(float(np.median(times)) * 1e6, 1), "unit": "us/step", "cores": oracle.threads(),
            "kind": "oracle",
            "sample": "whole workload (all sequences and heads, full context), routed step at tau 0.55, median of %d "
                      "runs; the dense step (routing off) took %.0f us once" % (len(times), dense_s * 1e6)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="c3", choices=["c0", "c1", "c2", "c3", "c4"])
    ap.add_argument("--also", default="c0,c1,c2,c4", help="comma list of further workloads to report ('' for none)")
    ap.add_argument("--copies", type=int, default=0, help="distinct K/V copies rotated through (0 = enough to defeat the last-level cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="leave out the seed sweep and the ragged / paged batches")
    ap.add_argument("--lean", action="store_true",
                    help="the run the profiler wraps: --workload only, no other workload, extras or CPU baseline")
    ap.add_argument("--num-splits", type=int, default=0, help="0 = balanced schedule, >0 = fixed Split-K chunks")
    ap.add_argument("--graph", action="store_true", help="also time the steps replayed from a captured HIP graph")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE_TOKENS",
                    help="run over a paged KV cache with this page size (power of two >= 64); 0 = contiguous")
    ap.add_argument("--timeline", default="", metavar="WORKLOADS",
                    help="per-phase accounting instead of the benchmark: comma list of workloads, needs the measurement "
                         "build (python -m paper_2604_16883_amd.build --timeline); prints markdown")
    ap.add_argument("--prefill-anchors", action="store_true",
                    help="--timeline: route on prefill-cached anchors and norms instead of row 0 of the key cache")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="instead of the benchmark: large batches of short contexts on the 8B-shaped layer (equal and ragged "
                         "lengths), routed and dense; prints a markdown table")
    ap.add_argument("--markdown", default="", metavar="PATH", help="also write the result tables as markdown to PATH")
    ap.add_argument("-v", "--verbose", action="store_true")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (KV groups are independent, so "
              "the path would shard by group across GPUs with no exchange; only N=1 is built)" % a.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if a.timeline:
        os.environ["SINKROUTER_LIB"] = os.path.join(ROOT, "paper_2604_16883_amd", "libsinkrouter_timeline.so")
    from paper_2604_16883_amd import binding, build
    if not a.timeline:
        build.ensure_built()
    binding.load()
    if a.lean:
        a.also, a.no_extras, a.no_cpu_baseline = "", True, True

    calib = hbm_calibration()
    if a.timeline:
        for name in a.timeline.split(","):
            for tau in ([TAU, 0.453, 2.0] if name == "c1" else [TAU, 2.0]):
                rep = timeline_report(name, tau, min(a.steps, 30), a.copies, a.prefill_anchors)
                print(timeline_markdown(rep, calib), flush=True)
                print("<!-- %s -->\n" % json.dumps(rep), flush=True)
                settle()
        return

    if a.batch_sweep:
        print(batch_sweep_markdown(a.steps, a.warmup), flush=True)
        return

    main_res, case = run_workload(a.workload, a.steps, a.warmup, a.copies, a.verbose, a.num_splits, a.paged, a.graph)
    cpu = None if a.no_cpu_baseline else cpu_baseline(case.sb)
    del case
    settle()
    others, extras, seeds, sweep = {}, {}, [], []
    for name in [x for x in a.also.split(",") if x and x != a.workload]:
        r, c2 = run_workload(name, a.steps, a.warmup, a.copies, a.verbose, a.num_splits, a.paged, a.graph)
        others[name] = r
        del c2
        settle()
    if not a.no_extras:
        from paper_2604_16883_amd import synth
        # the headline workload over its repetition seeds: the realised skip ratio is quantised by the 8 groups, and
        # the base seed is sparser (0.75) than the paper's operating point (~0.6, Section 5.1 / Appendix A)
        base = synth.WORKLOADS["c3"].base_seed
        for seed in range(base, base + 6):
            r, c2 = run_workload("c3", a.steps, a.warmup, a.copies, a.verbose, seed=seed, taus=False, prefill_anchors=False)
            rt = r["routed_tau0.55"]
            seeds.append({"seed": seed, **{k: rt[k] for k in ("skip_ratio", "algorithmic_bytes", "us_per_step", "partial_us", "combine_us",
                                                               "partial_frac_of_peak", "step_frac_of_peak")},
                          "dense_us_per_step": r["dense"]["us_per_step"]})
            if abs(rt["skip_ratio"] - 0.6) < 0.05 and "c3_skip0.625" not in extras:
                r["description"] += ", repetition seed %d: skip ratio %.3f, the paper's operating point" % (seed, rt["skip_ratio"])
                extras["c3_skip0.625"] = r
            del c2
            settle()
        # latency against context length on the headline shape (the paper's latency study, Section 5.3: gains are small
        # below 64K tokens and grow with the context), routed and dense on identical inputs
        for L in CONTEXT_SWEEP:
            r, c2 = run_workload("c3", a.steps, a.warmup, a.copies, a.verbose, seq_lens=[L], taus=False, prefill_anchors=False)
            rt, dn = r["routed_tau0.55"], r["dense"]
            sweep.append({"context": L, "skip_ratio": rt["skip_ratio"], "copies": r["copies"], "algorithmic_bytes": rt["algorithmic_bytes"],
                          "us_per_step": rt["us_per_step"], "step_frac_of_peak": rt["step_frac_of_peak"],
                          "dense_us_per_step": dn["us_per_step"], "dense_step_frac_of_peak": dn["step_frac_of_peak"],
                          "routed_vs_dense_speedup": r["routed_vs_dense_speedup"]})
            del c2
            settle()
        # one long and several short sequences, contiguous and paged: where the balanced schedule has to pay
        r, c2 = run_workload("c1", a.steps, a.warmup, a.copies, a.verbose, seq_lens=RAGGED_LENS, taus=False)
        extras["c1_ragged"] = r
        del c2
        settle()
        r, c2 = run_workload("c1", a.steps, a.warmup, a.copies, a.verbose, seq_lens=RAGGED_LENS, page_tokens=256, taus=False)
        r["description"] += ", paged (256-token pages, seeded random page order)"
        extras["c1_ragged_paged256"] = r
        del c2
        settle()

    routed = main_res["routed_tau0.55"]
    # the paged entry point has no per-kernel events: the whole step stands in for the kernel there
    achieved = routed["partial_GBps"] or routed["step_GBps"]
    dense_achieved = main_res["dense"]["partial_GBps"] or main_res["dense"]["step_GBps"]
    traffic, traffic_src = (None, "not the profiled configuration") if (a.num_splits or a.paged) else measured_traffic(a.workload, "routed_tau0.55")
    traffic_bytes = None if traffic is None else traffic["fetch_bytes"] + traffic["write_bytes"]
    line = {
        "metric": "decode-attention us/step (routed, tau=0.55) + effective HBM GB/s",
        "value": routed["us_per_step"],
        "unit": "us/step",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(routed["us_per_step"] / 1e3, 5),
        "timing": "device events around exactly `steps` calls, inside the synchronisation bracket",
        "us_per_step_host_clock": routed["us_per_step_host_clock"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic (seeded, sink-planted KV cache resident in HBM)",
        "config": {"workload": "%s: %s" % (a.workload, main_res["description"]), "kv_block": 64, "accumulate": "fp32",
                   "threshold": TAU, "skip_ratio": routed["skip_ratio"], "anchors": routed["anchors"],
                   "schedule": routed["schedule"], "partial_grid": routed["partial_grid"]},
        "roofline": {"bound": "hbm", "kernel": "sr_partial_balanced_kernel (routing probe fused)", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic_bytes,
                     "traffic_ratio": None if traffic_bytes is None else round(traffic_bytes / routed["algorithmic_bytes"], 4),
                     "traffic_source": traffic_src,
                     "algorithmic_bytes_per_launch": routed["algorithmic_bytes"],
                     "kernel_us": routed["partial_us"] or routed["us_per_step"],
                     "step_achieved": routed["step_GBps"], "step_frac": routed["step_frac_of_peak"],
                     "dense_achieved": dense_achieved, "dense_frac": round(dense_achieved / HBM_PEAK_GBS, 4),
                     "stream_read_probe_GBps": round(calib, 1)},
        "cpu_baseline": cpu,
        "dense_us_per_step": main_res["dense"]["us_per_step"],
        "routed_vs_dense_speedup": main_res["routed_vs_dense_speedup"],
        "us_per_step_prefill_anchors": main_res["routed_tau0.55_prefill_anchors"]["us_per_step"],
        # the metric is quoted at 128K and 512K: every workload's headline figures, same protocol
        "also": {name: headline(r) for name, r in {a.workload: main_res, **others, **extras}.items()},
        "seeds": seeds,
        "context_sweep": {"shape": "c3 (B1, 64/8 heads), tau 0.55", "points": sweep},
        "detail": {a.workload: main_res, **others, **extras},
    }
    if a.markdown:
        with open(a.markdown, "w") as f:
            f.write(results_markdown(line))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
