"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2604_16883_amd import synth

import gpu_util as gu


def _check(sb, taus=None, label="", **kw):
    G = sb.workload.group_size
    dev = None
    reports = []
    for tau in (taus or sb.taus):
        tc = (0, 0, 0, tau)
        res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=tc, dev=dev, **kw)
        dev = res["dev"]
        ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=tc, want_dense=True,
                            sm_scale=kw.get("sm_scale", 0.0), len_norm=kw.get("len_norm", 0.0),
                            routing_enabled=kw.get("routing_enabled", True))
        rep = gu.compare(res, ref, G, "%s tau=%.4f" % (label, tau))
        reports.append(rep)
        pl = res["plan"]
        print(label, "tau=%.4f" % tau, rep, "schedule", pl.schedule, "grid", pl.partial_grid, "splits", pl.num_splits,
              "chunk", pl.chunk_tokens, flush=True)
    return reports


# ---- reduced sizes: several tiles, ragged tails --------------------------------------------------
REDUCED = [
    ("c0", 4096, None),                       # the small config at its real size
    ("c1", 1000, [1000, 937, 64, 1]),         # ragged batch, tails inside a tile and a block
    ("c2", 3125, None),                       # G = 8, not a multiple of 64, secondary sinks
    ("c3", 2049, None),                       # G = 8, 64 query heads, one token past a block
    ("c4", 1500, [1500, 1217]),               # MHA (G = 1), image segments
]


@pytest.mark.parametrize("name,L,sl", REDUCED, ids=[r[0] for r in REDUCED])
def test_reduced_routed_and_dense(name, L, sl):
    w = synth.WORKLOADS[name].scaled(L)
    sb = synth.generate(w, seq_lens=sl, max_seq_len=L + (37 if sl else 0))
    reps = _check(sb, label=name + "-reduced")
    assert any(0 < r["skip_ratio"] < 1 for r in reps)
    _check(sb, taus=[0.55], label=name + "-reduced-dense", routing_enabled=False)


@pytest.mark.parametrize("num_splits", [1, 2, 3, 7, 64])
def test_output_independent_of_split_count(num_splits):
    w = synth.WORKLOADS["c0"].scaled(1733)
    sb = synth.generate(w, seed=11)
    _check(sb, label="splits=%d" % num_splits, num_splits=num_splits)


@pytest.mark.parametrize("Hq,Hkv", [(16, 1), (8, 4), (6, 2), (3, 3), (12, 1)])
def test_group_sizes(Hq, Hkv):
    w = synth.Workload("g", 2, Hq, Hkv, 777, 0.6, base_seed=50 + Hq)
    sb = synth.generate(w, seq_lens=[777, 300])
    _check(sb, label="Hq%d/Hkv%d" % (Hq, Hkv))


def test_large_batches_take_the_unfused_and_fixed_paths():
    # more than 256 query heads in the batch: separate probe kernel + balanced schedule
    w = synth.Workload("wide", 20, 32, 8, 300, 0.6, base_seed=91)
    sb = synth.generate(w, seq_lens=[300 - 7 * b for b in range(20)])
    reps = _check(sb, label="B20 (unfused probe)")
    assert 0 < reps[0]["skip_ratio"] < 1
    # more than 256 query heads but at most 64 groups: separate probe kernel + schedule built in registers
    w = synth.Workload("wide_groups", 40, 16, 1, 260, 0.6, base_seed=95)
    sb = synth.generate(w, seq_lens=[260 - 6 * b for b in range(40)])
    reps = _check(sb, label="B40 G16 (unfused probe, 40 groups)")
    assert 0 < reps[0]["skip_ratio"] < 1
    # exactly 256 query heads: the fused probe sweeps twice; one head more: the separate probe
    w = synth.Workload("fused256", 8, 32, 8, 200, 0.6, base_seed=93)
    sb = synth.generate(w, seq_lens=[200 - 11 * (b % 9) for b in range(8)])
    reps = _check(sb, label="B8 (fused probe, 256 heads)")
    assert 0 < reps[0]["skip_ratio"] < 1
    w = synth.Workload("unfused272", 17, 16, 4, 200, 0.6, base_seed=96)
    sb = synth.generate(w, seq_lens=[200 - 9 * (b % 11) for b in range(17)])
    reps = _check(sb, label="B17 (separate probe, 272 heads)")
    assert 0 < reps[0]["skip_ratio"] < 1
    # 2000 (sequence, group) pairs: the schedule scan runs eight rounds
    w = synth.Workload("scan", 250, 16, 8, 100, 0.6, base_seed=94)
    sb = synth.generate(w, seq_lens=[100 - (b % 41) for b in range(250)])
    res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens)
    assert res["plan"].schedule == 1
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True)
    print("B250", gu.compare(res, ref, 2, "B250 (balanced, 2000 groups)"), flush=True)
    # more than 2048 (sequence, group) pairs: falls back to fixed chunks
    w = synth.Workload("many", 300, 16, 8, 130, 0.6, base_seed=92)
    sb = synth.generate(w, seq_lens=[130 - (b % 67) for b in range(300)])
    res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens)
    assert res["plan"].schedule == 0
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True)
    rep = gu.compare(res, ref, 2, "B300 (fixed fallback)")
    print("B300", rep, flush=True)
    assert 0 < rep["skip_ratio"] < 1


@pytest.mark.parametrize("empty", [0, 1, 2], ids=["130-active", "128-active", "126-active"])
def test_both_sides_of_the_share_scheme_switch(empty):
    """130 (sequence, group) pairs, routing off, `empty` sequences of length 0: 130 Active Groups take contiguous
    shares (more than half as many as workgroups), 128 and 126 take per-group shares, built in LDS (more than 64
    groups).  Ragged lengths, so the groups get different numbers of workgroups."""
    B, Hq, Hkv, L = 65, 4, 2, 700
    lens = [L - 9 * (b % 23) for b in range(B)]
    for b in range(empty):
        lens[7 + 11 * b] = 0
    w = synth.Workload("switch", B, Hq, Hkv, L, 0.5, base_seed=300 + empty, planted_per_head=4)
    sb = synth.generate(w, seq_lens=lens)
    for kw in (dict(routing_enabled=False), dict(tau_coef=(0, 0, 0, 0.55))):
        res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, **kw)
        ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True, **kw)
        rep = gu.compare(res, ref, w.group_size, "switch %d %s" % (empty, kw))
        print("switch", empty, kw, rep, flush=True)
        assert res["plan"].schedule == 1


@pytest.mark.parametrize("shape", ["narrow", "wide-fixed", "wide-balanced"])
def test_heads_with_more_records_than_one_merge_sweep(shape):
    """The merge kernel takes a head's records in sweeps (64 records with the narrow workgroup shape, 256 with the
    wide one, whose four column parts of a head must also line up).  narrow: 18 (sequence, group) pairs of which one
    sequence's two are non-empty, so each gets 127 of the 256 workgroups, which take 2 blocks each: 100 records per
    head, two sweeps.
    wide-fixed: 300 fixed chunks of 256 tokens, one group: two sweeps.  wide-balanced: one group on all 256 shares."""
    if shape == "narrow":
        B, Hq, Hkv, L = 9, 8, 2, 64 * 200
        lens = [0] * B
        lens[4] = L - 5
        kw, records = dict(), 100
    elif shape == "wide-fixed":
        B, Hq, Hkv, L = 1, 4, 1, 256 * 300
        lens, kw, records = [L - 3], dict(num_splits=300), 300
    else:
        B, Hq, Hkv, L = 1, 4, 1, 64 * 700
        lens, kw, records = [L - 70], dict(), 233     # 699 blocks over 255 workgroups: shares of 3 blocks
    w = synth.Workload("sweeps", B, Hq, Hkv, L, 0.5, base_seed=410, planted_per_head=4)
    sb = synth.generate(w, seq_lens=lens)
    res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, routing_enabled=False, **kw)
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True, routing_enabled=False)
    rep = gu.compare(res, ref, w.group_size, "sweeps " + shape)
    print("sweeps", shape, rep, res["plan"].schedule, res["plan"].slots_per_head, flush=True)
    assert res["plan"].slots_per_head >= records


def test_equal_groups_whose_own_shares_would_leave_half_the_chip_idle():
    """128 equally long (sequence, group) pairs, routing off: per-group shares would be one workgroup each (128 of 256
    busy), so the schedule falls back to contiguous shares (two workgroups per group); 100 such pairs keep their own
    shares (two each).  Both are built in LDS (more than 64 groups)."""
    import bench
    for B in (64, 50):
        Hq, Hkv, L = 4, 2, 700
        w = synth.Workload("cliff", B, Hq, Hkv, L, 0.5, base_seed=520 + B, planted_per_head=4)
        sb = synth.generate(w)
        assert bench.per_group_shares([(L + 63) // 64] * (B * Hkv), 256) == (B == 50)
        res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, routing_enabled=False)
        ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True, routing_enabled=False)
        rep = gu.compare(res, ref, w.group_size, "cliff B=%d" % B)
        print("cliff", B, rep, flush=True)
        assert res["plan"].schedule == 1


def test_edge_lengths():
    # lengths 0 and 1, exactly one block, one block + 1, all with a poisoned tail beyond seq_len
    w = synth.Workload("edge", 6, 8, 2, 300, 0.5, base_seed=77)
    sl = [0, 1, 64, 65, 256, 257]
    sb = synth.generate(w, seq_lens=sl, max_seq_len=300)
    for tau in (0.55, -2.0, 2.0):
        res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=(0, 0, 0, tau))
        ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=(0, 0, 0, tau), want_dense=True)
        rep = gu.compare(res, ref, 4, "edge tau=%g" % tau)
        print("edge", tau, rep, flush=True)
        assert res["mask"][0].tolist() == [0, 0]             # empty sequence: never a Sink Group
        assert np.all(res["out_bits"][0] == 0)
    # L = 1 and active: out = V_0 exactly (already bf16)
    res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, routing_enabled=False)
    for h in range(8):
        assert np.array_equal(res["out_bits"][1, h], sb.v[1, h // 4, 0])


def test_lengths_outside_the_cache_are_clamped_on_the_device():
    """seq_lens below 0 or above the cache stride: the device clamps them to [0, L_max] before the
    threshold, the schedule and the attention use them.  The caches hold NaN patterns wherever the
    clamped length says no valid row is, the threshold depends on the length (so a clamp that missed
    tau would flip decisions: unclamped, the huge lengths give tau far below -1), and every path that
    reads a length is taken: fused probe + balanced schedule, fixed chunks + separate probe, paged."""
    from test_gpu_paged import run_paged
    Lmax = 300
    given = [-5, 0, Lmax + 17, Lmax, 131, -2 ** 31, 2 ** 31 - 1, 1]
    valid = [0, 0, Lmax, Lmax, 131, 0, Lmax, 1]
    w = synth.Workload("clamp", len(given), 8, 2, Lmax, 0.5, base_seed=78)
    sb = synth.generate(w, seq_lens=valid, max_seq_len=Lmax)
    kw = dict(tau_coef=(0.0, 0.0, -0.3, 0.85), len_norm=float(Lmax))          # tau(L_max) = 0.55
    ref = oracle.decode(sb.q, sb.k, sb.v, given, want_dense=True, **kw)
    same = oracle.decode(sb.q, sb.k, sb.v, valid, want_dense=True, **kw)
    assert np.array_equal(ref.mask, same.mask) and np.array_equal(ref.out, same.out) and np.array_equal(ref.tau, same.tau)
    assert 0 < ref.mask.mean() < 1
    results = []
    for extra in (dict(), dict(num_splits=3), dict(routing_enabled=False)):
        print("clamp", extra, flush=True)
        r = ref if extra.get("routing_enabled", True) else oracle.decode(sb.q, sb.k, sb.v, given, want_dense=True,
                                                                         routing_enabled=False, **kw)
        res = gu.run_hip(sb.q, sb.k, sb.v, given, **kw, **extra)
        rep = gu.compare(res, r, w.group_size, "clamp %s" % extra)
        print("clamp", extra, rep, flush=True)
        for b in (0, 1, 5):
            assert np.all(res["out_bits"][b] == 0) and not res["mask"][b].any()
        results.append(res)
    kp, table = synth.to_pages(sb.k, valid, 64, seed=5)
    vp, _ = synth.to_pages(sb.v, valid, 64, seed=5)
    for extra, cont in ((dict(), results[0]), (dict(num_splits=3), results[1])):
        print("clamp paged", extra, flush=True)
        pres = run_paged(sb, kp, vp, table, 64, given_lens=given, **kw, **extra)
        assert np.array_equal(pres["out_bits"], cont["out_bits"]) and np.array_equal(pres["mask"], cont["mask"])
    # a wide batch (more than 512 query heads): the separate probe kernel and the LDS-built schedule
    B = 70
    given = [(-7, 0, 200 + 9, 200, 77, 2 ** 31 - 1, -2 ** 31)[b % 7] for b in range(B)]
    valid = [min(max(x, 0), 200) for x in given]
    w = synth.Workload("clamp_wide", B, 8, 2, 200, 0.5, base_seed=79, planted_per_head=4)
    sb = synth.generate(w, seq_lens=valid, max_seq_len=200)
    kw = dict(tau_coef=(0.0, 0.0, -0.3, 0.85), len_norm=200.0)
    ref = oracle.decode(sb.q, sb.k, sb.v, given, want_dense=True, **kw)
    res = gu.run_hip(sb.q, sb.k, sb.v, given, **kw)
    print("clamp wide", gu.compare(res, ref, w.group_size, "clamp wide"), flush=True)


def test_threshold_cubic_scale_and_cached_norm():
    w = synth.WORKLOADS["c1"].scaled(900, batch=3)
    sb = synth.generate(w, seed=5, seq_lens=[900, 450, 200])
    coef = (0.4, -0.9, 0.5, 0.45)
    kw = dict(tau_coef=coef, len_norm=900.0, sm_scale=0.11)
    res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, **kw)
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True, **kw)
    print("cubic", gu.compare(res, ref, 4, "cubic"), ref.tau, flush=True)
    assert len(set(np.round(ref.tau, 6))) == 3
    # cached anchor norm (Section 4.1): passing the true norm changes nothing; a doubled norm halves S
    kn = np.linalg.norm(synth.bf16_bits_to_f32(sb.k[:, :, 0]).astype(np.float64), axis=-1)
    res1 = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, k0_norm=kn, **kw)
    np.testing.assert_allclose(res1["score"], res["score"], rtol=0, atol=1e-6)
    res2 = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, k0_norm=2 * kn, **kw)
    ref2 = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True, k0_norm=2 * kn, **kw)
    gu.compare(res2, ref2, 4, "doubled-norm")


def test_mask_reads_token0_only_and_skip_bound():
    w = synth.WORKLOADS["c0"].scaled(1024)
    sb = synth.generate(w, seed=3)
    base = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens)
    k2, v2 = sb.k.copy(), sb.v.copy()
    rng = np.random.default_rng(1)
    k2[:, :, 1:] = rng.integers(0, 0x4000, size=k2[:, :, 1:].shape, dtype=np.uint16)
    v2[:] = rng.integers(0, 0x4000, size=v2.shape, dtype=np.uint16)
    alt = gu.run_hip(sb.q, k2, v2, sb.seq_lens)
    assert np.array_equal(alt["mask"], base["mask"])
    assert np.array_equal(alt["score"], base["score"])
    # Eq. 4 on the GPU's dense output: ||u|| <= alpha_0 ||v_0|| + (1 - alpha_0) max ||v_t||
    dense = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, routing_enabled=False)
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True)
    vf = synth.bf16_bits_to_f32(sb.v).astype(np.float64)
    for h in range(w.n_q_heads):
        g = h // w.group_size
        bound = ref.alpha0[0, h] * np.linalg.norm(vf[0, g, 0]) + (1 - ref.alpha0[0, h]) * np.linalg.norm(vf[0, g, 1:], axis=-1).max()
        assert np.linalg.norm(dense["out"][0, h]) <= bound + 1e-2


# ---- full sizes, in the launch configuration the benchmark times -----------------------------------
@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4"])
def test_full_size(name):
    w = synth.WORKLOADS[name]
    sb = synth.generate(w)
    print(name, "generated", sb.k.nbytes * 2 / 1e6, "MB", flush=True)
    _check(sb, label=name + "-full")
    _check(sb, taus=[0.55], label=name + "-full-dense", routing_enabled=False)
    _check(sb, taus=[0.55], label=name + "-full-fixed-chunks", num_splits=200)


# ---- the longest cache the library accepts ---------------------------------------------------------
def test_maximum_sequence_length():
    """max_seq_len = 2^24 tokens (the documented limit), one KV group of two heads: 8.6 GB of K and V.
    Exercises the 64-bit row offsets and the 32-bit token arithmetic at their largest values; the
    length is one short of the stride so the tail is ragged too."""
    import time
    L = (1 << 24) - 1
    w = synth.Workload("max_len", 1, 2, 1, L, 0.5, base_seed=7000, planted_per_head=16)
    t0 = time.time()
    sb = synth.generate(w, max_seq_len=1 << 24)
    print("max_len generated in %.1f s" % (time.time() - t0), flush=True)
    res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=(0, 0, 0, 2.0))
    print("max_len gpu done", flush=True)
    t0 = time.time()
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=(0, 0, 0, 2.0), want_dense=True)
    print("max_len oracle %.1f s" % (time.time() - t0), flush=True)
    rep = gu.compare(res, ref, 2, "max_len")
    pl = res["plan"]
    assert pl.schedule == 1 and pl.slots_per_head == 257
    assert not res["mask"].any()
    print("max_len", rep, flush=True)


def test_maximum_group_count():
    """65535 (sequence, KV group) pairs, the documented limit (fixed chunks, separate probe kernel),
    with ragged lengths 0..70 on plain Gaussian data: about half the groups are Sink Groups at tau = 0."""
    B, L = 65535, 70
    lens = (np.arange(B) * 37) % (L + 1)
    q, k, v, sl = synth.random_small(7100, B, 1, 1, 128, L, lens)
    res = gu.run_hip(q, k, v, sl, tau_coef=(0, 0, 0, 0.0))
    assert res["plan"].schedule == 0 and res["plan"].partial_grid == B * res["plan"].num_splits
    ref = oracle.decode(q, k, v, sl, tau_coef=(0, 0, 0, 0.0), want_dense=True)
    rep = gu.compare(res, ref, 1, "65535 groups")
    print("65535 groups", rep, flush=True)
    assert 0.3 < rep["skip_ratio"] < 0.7


def test_degenerate_routing_inputs():
    """The degenerate cases of the routing rule, where the decision must be exact and not merely
    within the band: a zero anchor or zero query (cosine 0, not NaN), an exact tie S == tau (strict
    comparison keeps the group active), a cached norm of zero, and a NaN anchor (group stays active)."""
    B, Hq, Hkv, L = 1, 8, 4, 200
    q, k, v, sl = synth.random_small(7200, B, Hq, Hkv, 128, L)
    k = k.copy()
    q = q.copy()
    k[0, 0, 0] = 0                       # group 0: K_0 = 0  -> every cosine 0, S = 0 exactly
    q[0, 2] = 0                          # group 1, first head: q = 0 -> its cosine is 0
    q[0, 4] = k[0, 2, 0]                 # group 2: both heads equal the anchor -> S = 1 up to rounding
    q[0, 5] = k[0, 2, 0]
    for tau, want0 in ((0.0, 0), (-1e-6, 1)):          # tie at S == tau == 0: active; just below: Sink Group
        res = gu.run_hip(q, k, v, sl, tau_coef=(0, 0, 0, tau))
        ref = oracle.decode(q, k, v, sl, tau_coef=(0, 0, 0, tau), want_dense=True)
        assert res["score"][0, 0] == 0.0 and ref.group_score[0, 0] == 0.0
        assert res["mask"][0, 0] == want0 == ref.mask[0, 0]
        assert np.isfinite(res["score"]).all()
        gu.compare(res, ref, 2, "degenerate tau=%g" % tau)
    res = gu.run_hip(q, k, v, sl, tau_coef=(0, 0, 0, 0.999))
    ref = oracle.decode(q, k, v, sl, tau_coef=(0, 0, 0, 0.999), want_dense=True)
    assert res["mask"][0].tolist() == [0, 0, 1, 0] == ref.mask[0].tolist()
    np.testing.assert_allclose(res["score"][0, 1], 0.5 * ref.head_cos[0, 3], rtol=0, atol=2e-6)   # the zero query counts as 0
    # cached norm of zero: the denominator vanishes, cosines are 0, nothing exceeds tau = 0
    zero = np.zeros((B, Hkv), np.float32)
    res = gu.run_hip(q, k, v, sl, tau_coef=(0, 0, 0, 0.0), k0_norm=zero)
    ref = oracle.decode(q, k, v, sl, tau_coef=(0, 0, 0, 0.0), k0_norm=zero, want_dense=True)
    assert not res["mask"].any() and not ref.mask.any() and np.all(res["score"] == 0.0)
    gu.compare(res, ref, 2, "zero cached norm")
    # NaN in a separately cached anchor whose cached norm is finite: the dot product and so the score
    # are NaN, the comparison is false, the group stays active.  (Without a cached norm the norm is
    # NaN too, the denominator test fails and the cosine is 0, on both sides.)
    import torch
    k0 = k[:, :, 0].copy()
    k0[0, 3, 7] = 0x7FC0
    k0_dev = gu.to_dev(k0)
    kn = np.linalg.norm(synth.bf16_bits_to_f32(k[:, :, 0]).astype(np.float64), axis=-1)
    kn[0, 0] = 1.0
    res = gu.run_hip(q, k, v, sl, tau_coef=(0, 0, 0, -2.0), k0=k0_dev, k0_norm=kn)
    ref = oracle.decode(q, k, v, sl, tau_coef=(0, 0, 0, -2.0), k0=k0, k0_norm=kn, want_dense=True)
    assert res["mask"][0].tolist() == [1, 1, 1, 0] == ref.mask[0].tolist()
    assert np.isnan(res["score"][0, 3]) and np.isnan(ref.group_score[0, 3])
    assert np.all(res["out_bits"][0, :6] == 0)
    err = np.abs(res["out"][0, 6:].astype(np.float64) - ref.out[0, 6:])
    assert err.max() <= gu.MAX_ABS_TOL
    res = gu.run_hip(q, k, v, sl, tau_coef=(0, 0, 0, -2.0), k0=k0_dev)
    ref = oracle.decode(q, k, v, sl, tau_coef=(0, 0, 0, -2.0), k0=k0, want_dense=True)
    assert res["mask"][0].tolist() == [1, 1, 1, 1] == ref.mask[0].tolist()
    assert res["score"][0, 3] == 0.0 == ref.group_score[0, 3]
    torch.cuda.synchronize()


def test_threshold_inside_the_rounding_band():
    """A threshold closer to a group's score than fp32 can resolve: either decision is accepted for
    that group, it is counted, and the output must match the oracle's under the decision the GPU
    took (zeros, or the dense result)."""
    w = synth.WORKLOADS["c0"].scaled(1000)
    sb = synth.generate(w, seed=11)
    scores = oracle.route(sb.q, sb.k, sb.seq_lens).group_score[0]
    hits = 0
    for g in range(w.n_kv_heads):
        for delta in (-2e-8, 2e-8):
            tau = float(scores[g] + delta)
            res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=(0, 0, 0, tau))
            ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=(0, 0, 0, tau), want_dense=True)
            rep = gu.compare(res, ref, w.group_size, "band g%d %+g" % (g, delta))
            assert rep["near_threshold"] >= 1
            hits += rep["mask_disagree_in_band"]
    print("in-band disagreements:", hits, "of", 2 * w.n_kv_heads, flush=True)
