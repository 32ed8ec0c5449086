"""Seeded random sweep of shapes, ragged lengths, thresholds, schedules and cache layouts: HIP path vs
the CPU oracle (needs an MI355X).  Sizes are small so the oracle stays fast; every case is printed."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2604_16883_amd import synth

import gpu_util as gu
from test_gpu_paged import run_paged

GROUPINGS = [(1, 1), (2, 1), (4, 2), (8, 2), (32, 8), (16, 16), (40, 40), (5, 5), (24, 3), (16, 1), (14, 2), (64, 8)]


N_CASES = int(os.environ.get("SR_RANDOM_CASES", "36"))     # a longer sweep: SR_RANDOM_CASES=600 pytest ...


@pytest.mark.parametrize("case", range(N_CASES))
def test_random_case(case):
    rng = np.random.default_rng(10_000 + case)
    Hq, Hkv = GROUPINGS[case % len(GROUPINGS)]
    B = int(rng.integers(1, 6))
    Lmax = int(rng.choice([1, 3, 63, 64, 65, 127, 255, 256, 257, 300, 511, 777, 1024, 1500, 2049]))
    sl = [int(rng.integers(0, Lmax + 1)) if rng.random() < 0.7 else Lmax for _ in range(B)]
    sl[int(rng.integers(0, B))] = Lmax                       # at least one full-length sequence
    stride = Lmax + int(rng.integers(0, 40))
    w = synth.Workload("rnd", B, Hq, Hkv, Lmax, float(rng.uniform(0.3, 0.8)), base_seed=case,
                       secondary_sinks=int(rng.integers(0, 3)), image_segments=0)
    sb = synth.generate(w, seed=case, seq_lens=sl, max_seq_len=stride)
    tau = float(np.float32(rng.uniform(0.2, 0.8)))
    kw = dict(tau_coef=(0, 0, 0, tau))
    mode = case % 4
    if mode == 1:
        kw["num_splits"] = int(rng.integers(1, 9))
    if mode == 2:
        kw["sm_scale"] = float(np.float32(rng.uniform(0.05, 0.15)))
    if mode == 3:
        kw.update(tau_coef=(0.0, float(np.float32(rng.uniform(-0.3, 0.3))), 0.0, tau), len_norm=float(stride))
    okw = {k: v for k, v in kw.items() if k != "num_splits"}
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True, **okw)
    res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, **kw)
    rep = gu.compare(res, ref, w.group_size, "case %d" % case)
    print("case", case, dict(B=B, Hq=Hq, Hkv=Hkv, Lmax=Lmax, stride=stride, sl=sl, **kw), rep, flush=True)
    if case % 3 == 0 and stride >= 1:                        # the same inputs through the paged entry point
        pt = int(rng.choice([64, 128, 512]))
        kp, tab = synth.to_pages(sb.k, sb.seq_lens, pt, seed=case)
        vp, _ = synth.to_pages(sb.v, sb.seq_lens, pt, seed=case)
        pres = run_paged(sb, kp, vp, tab, pt, **kw)
        assert np.array_equal(pres["out_bits"], res["out_bits"]) and np.array_equal(pres["mask"], res["mask"])


N_WIDE = int(os.environ.get("SR_RANDOM_WIDE_CASES", "24"))


@pytest.mark.parametrize("case", range(N_WIDE))
def test_random_wide_batches(case):
    """Larger batches: both sides of the 512-head limit of the fused probe and of the 64-group limit of
    the register-built schedule, short ragged sequences."""
    rng = np.random.default_rng(20_000 + case)
    Hq, Hkv = [(16, 1), (32, 8), (8, 8), (12, 2), (64, 8), (4, 1)][case % 6]
    B = int(rng.choice([3, 9, 17, 33, 48, 70]))
    Lmax = int(rng.choice([64, 130, 257, 400]))
    sl = [int(rng.integers(0, Lmax + 1)) for _ in range(B)]
    sl[int(rng.integers(0, B))] = Lmax
    w = synth.Workload("wide_rnd", B, Hq, Hkv, Lmax, float(rng.uniform(0.3, 0.8)), base_seed=500 + case, planted_per_head=4)
    sb = synth.generate(w, seed=500 + case, seq_lens=sl)
    tau = float(np.float32(rng.uniform(0.3, 0.7)))
    kw = dict(tau_coef=(0, 0, 0, tau))
    if case % 5 == 4:
        kw["num_splits"] = int(rng.integers(1, 4))
    okw = {k: v for k, v in kw.items() if k != "num_splits"}
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True, **okw)
    res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, **kw)
    rep = gu.compare(res, ref, w.group_size, "wide case %d" % case)
    print("wide", case, dict(B=B, Hq=Hq, Hkv=Hkv, Lmax=Lmax, heads=B * Hq, groups=B * Hkv, **kw), rep, flush=True)
