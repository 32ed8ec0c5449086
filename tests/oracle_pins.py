"""Pins of the CPU oracle: checks against things other than the oracle itself.

Every function takes ``lib`` (None = the real oracle, else the path of another
build of it) so that the mutation test can run the same pins on deliberately
broken copies and show that each planted mistake is caught.

What fixes the expected values:
  * hand-computed fixtures (tests/golden/hand_cases.json);
  * scipy/numpy library routines (softmax, logsumexp, einsum) on fp64 copies of
    the inputs with the KV heads explicitly repeated per query head;
  * closed forms and invariances that follow from Section 3 Eq. 1, Eq. 3-5 and
    Section 4.2 Eq. 11-14 of the paper.
"""
from __future__ import annotations

import json
import os

import numpy as np
from scipy.special import logsumexp, softmax

import oracle
from paper_2604_16883_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "hand_cases.json")


def bits(x):
    b = synth.f32_to_bf16_bits(np.asarray(x, np.float32))
    # the fixtures and hand-made cases must be exactly representable
    assert np.array_equal(synth.bf16_bits_to_f32(b), np.asarray(x, np.float32))
    return b


def f64(b):
    return synth.bf16_bits_to_f32(b).astype(np.float64)


def library_attention(q, k, v, seq_lens, sm_scale=0.0):
    """Dense attention from library routines, KV heads repeated per query head."""
    qf, kf, vf = f64(q), f64(k), f64(v)
    B, Hq, D = qf.shape
    Hkv = kf.shape[1]
    r = Hq // Hkv
    kf = np.repeat(kf, r, axis=1)
    vf = np.repeat(vf, r, axis=1)
    scale = sm_scale if sm_scale != 0.0 else 1.0 / np.sqrt(D)
    out = np.zeros((B, Hq, D))
    lse = np.full((B, Hq), -np.inf)
    a0 = np.full((B, Hq), np.nan)
    for b in range(B):
        L = int(seq_lens[b])
        if L == 0:
            continue
        z = np.einsum("hd,htd->ht", qf[b], kf[b, :, :L]) * scale
        p = softmax(z, axis=-1)
        out[b] = np.einsum("ht,htd->hd", p, vf[b, :, :L])
        lse[b] = logsumexp(z, axis=-1)
        a0[b] = p[:, 0]
    return out, lse, a0


# --------------------------------------------------------------------------------------------
def check_golden(lib=None):
    cases = json.load(open(GOLDEN))["cases"]
    assert len(cases) >= 8
    for c in cases:
        q = bits(c["q"])[None]
        k = bits(c["k"])[None]
        v = bits(c["v"])[None]
        L = c["seq_len"]
        r = oracle.decode(q, k, v, [L], tau_coef=c.get("tau_coef", (0, 0, 0, 0.55)),
                          len_norm=c.get("len_norm", 0.0), sm_scale=c["sm_scale"],
                          routing_enabled=bool(c["routing_enabled"]), want_dense=True, libpath=lib)
        tol = dict(rtol=0, atol=1e-14)
        np.testing.assert_allclose(r.out[0], np.array(c["expect_out"]), err_msg=c["name"], **tol)
        if "expect_alpha0" in c:
            np.testing.assert_allclose(r.alpha0[0], c["expect_alpha0"], err_msg=c["name"], **tol)
        if "expect_lse" in c:
            np.testing.assert_allclose(r.lse[0], c["expect_lse"], err_msg=c["name"], **tol)
        if "expect_head_cos" in c:
            np.testing.assert_allclose(r.head_cos[0], c["expect_head_cos"], err_msg=c["name"], **tol)
        if "expect_group_score" in c:
            np.testing.assert_allclose(r.group_score[0], c["expect_group_score"], err_msg=c["name"], **tol)
        if "expect_tau" in c:
            np.testing.assert_allclose(r.tau[0], c["expect_tau"], err_msg=c["name"], **tol)
        if "expect_mask" in c:
            assert r.mask[0].tolist() == c["expect_mask"], c["name"]


def check_brute_force_dense(lib=None):
    """Routing disabled == library softmax attention (several tiny shapes, GQA and MHA, ragged)."""
    shapes = [(1, 1, 1, 4, 1), (2, 4, 2, 8, 16), (2, 6, 2, 8, 13), (1, 4, 4, 6, 9), (3, 8, 1, 4, 7)]
    for i, (B, Hq, Hkv, D, L) in enumerate(shapes):
        sl = [max(1, L - 3 * b) for b in range(B)]
        q, k, v, sl = synth.random_small(100 + i, B, Hq, Hkv, D, L, sl, scale=1.5)
        for scale in (0.0, 0.37):
            r = oracle.decode(q, k, v, sl, routing_enabled=False, sm_scale=scale, want_dense=True, libpath=lib)
            out, lse, a0 = library_attention(q, k, v, sl, scale)
            np.testing.assert_allclose(r.out, out, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(r.dense_out, out, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(r.lse, lse, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(r.alpha0, a0, rtol=1e-12, atol=1e-14)
            assert not r.mask.any()


def check_routed_vs_library(lib=None):
    """Routed output == library attention on active groups, exact zeros on sink groups;
    the mask equals a numpy evaluation of the cosine / mean / strict compare."""
    for seed in range(6):
        B, Hq, Hkv, D, L = 2, 8, 2, 8, 12
        q, k, v, sl = synth.random_small(200 + seed, B, Hq, Hkv, D, L, [L, L - 5])
        # make the first group of each sequence sink-like: heads aligned with K_0
        kf = synth.bf16_bits_to_f32(k)
        qf = synth.bf16_bits_to_f32(q)
        r_ = Hq // Hkv
        for b in range(B):
            qf[b, :r_] = qf[b, :r_] * 0.25 + 2.0 * kf[b, 0, 0]
        q = synth.f32_to_bf16_bits(qf)
        tau = 0.3 + 0.05 * seed
        r = oracle.decode(q, k, v, sl, tau_coef=(0, 0, 0, tau), want_dense=True, libpath=lib)
        out, _, _ = library_attention(q, k, v, sl)
        qd, kd = f64(q), f64(k)
        cos = np.zeros((B, Hq))
        for b in range(B):
            for h in range(Hq):
                a, c = qd[b, h], kd[b, h // r_, 0]
                cos[b, h] = a @ c / (np.linalg.norm(a) * np.linalg.norm(c))
        S = cos.reshape(B, Hkv, r_).mean(-1)
        np.testing.assert_allclose(r.head_cos, cos, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(r.group_score, S, rtol=1e-13, atol=1e-15)
        mask = (S > tau).astype(np.uint8)
        assert np.array_equal(r.mask, mask)
        assert mask.any() and not mask.all()
        keep = np.repeat(1 - mask, r_, axis=1)[..., None]
        np.testing.assert_allclose(r.out, out * keep, rtol=1e-12, atol=1e-13)
        assert np.all(r.out[np.repeat(mask, r_, axis=1).astype(bool)] == 0.0)
        np.testing.assert_allclose(r.dense_out, out, rtol=1e-12, atol=1e-13)


def check_splitk_equals_single_pass(lib=None):
    """Split-K partials + log-sum-exp merge == single pass, for many split lists."""
    rng = np.random.default_rng(7)
    B, Hq, Hkv, D, L = 2, 4, 2, 8, 37
    q, k, v, sl = synth.random_small(300, B, Hq, Hkv, D, L, [L, 20], scale=2.0)
    ref = oracle.decode(q, k, v, sl, routing_enabled=False, libpath=lib)
    lists = [[0, L], [0, 1, L], [0, 0, 5, 5, L], [0, 20, L], [0, 36, 37, 60], list(range(0, L + 1)),
             [0, 64, 128]]
    for _ in range(10):
        n = int(rng.integers(1, 9))
        cuts = np.sort(rng.integers(0, L + 1, size=n - 1)).tolist()
        lists.append([0] + cuts + [L])
    for bnd in lists:
        out, mask, pm, pl = oracle.decode_splitk(q, k, v, sl, bnd, routing_enabled=False, libpath=lib)
        np.testing.assert_allclose(out, ref.out, rtol=1e-12, atol=1e-13, err_msg=str(bnd))
        # merged statistics reproduce the log-sum-exp of the whole row
        with np.errstate(divide="ignore"):
            lse = logsumexp(pm + np.log(pl), axis=-1)
        np.testing.assert_allclose(lse, ref.lse, rtol=1e-12, atol=1e-12, err_msg=str(bnd))
        # an empty chunk is (m=-inf, l=0)
        for b in range(B):
            for j in range(len(bnd) - 1):
                if min(bnd[j + 1], sl[b]) <= min(bnd[j], sl[b]):
                    assert np.all(np.isneginf(pm[b, :, j])) and np.all(pl[b, :, j] == 0)


def check_closed_forms(lib=None):
    D = 4
    # L = 1: out = V_0 whatever q, K are
    q, k, v, sl = synth.random_small(400, 1, 2, 1, D, 1)
    r = oracle.decode(q, k, v, sl, routing_enabled=False, libpath=lib)
    np.testing.assert_array_equal(r.out[0, 0], f64(v)[0, 0, 0])
    np.testing.assert_array_equal(r.out[0, 1], f64(v)[0, 0, 0])
    # one key far above the rest: out = that value row (weights of the others < e^-64)
    L = 9
    q, k, v, sl = synth.random_small(401, 1, 1, 1, D, L, scale=0.25)
    qf = synth.bf16_bits_to_f32(q)
    kf = synth.bf16_bits_to_f32(k)
    kf[0, 0, 5] = 256.0 * qf[0, 0]
    k2 = synth.f32_to_bf16_bits(kf)
    assert f64(q)[0, 0] @ f64(q)[0, 0] > 0.05
    r = oracle.decode(q, k2, v, sl, routing_enabled=False, sm_scale=8.0, libpath=lib)
    np.testing.assert_allclose(r.out[0, 0], f64(v)[0, 0, 5], rtol=0, atol=1e-15)
    # shift invariance: adding c*e_1 to every key with q = 2*e_1 shifts all scores by 2c
    qs = bits(np.array([[[2.0, 0.0, 0.0, 0.0]]]))
    kk = np.round(np.random.default_rng(3).standard_normal((1, 1, L, D)) * 4) / 4
    vv = np.round(np.random.default_rng(4).standard_normal((1, 1, L, D)) * 4) / 4
    k_a = bits(kk)
    kk2 = kk.copy()
    kk2[..., 0] += 3.0
    k_b = bits(kk2)
    ra = oracle.decode(qs, k_a, bits(vv), [L], routing_enabled=False, sm_scale=0.5, want_dense=True, libpath=lib)
    rb = oracle.decode(qs, k_b, bits(vv), [L], routing_enabled=False, sm_scale=0.5, want_dense=True, libpath=lib)
    np.testing.assert_allclose(ra.out, rb.out, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(rb.lse - ra.lse, 3.0, rtol=0, atol=1e-13)
    # seq_len 0: zero output, mask 0, even with a threshold everything exceeds
    q, k, v, sl = synth.random_small(402, 2, 2, 1, D, 5, [0, 5])
    r = oracle.decode(q, k, v, sl, tau_coef=(0, 0, 0, -2.0), libpath=lib)
    assert np.all(r.out[0] == 0) and r.mask[0, 0] == 0 and r.mask[1, 0] == 1
    # a length above the cache stride is clamped to it
    q, k, v, sl = synth.random_small(403, 1, 2, 1, D, 6)
    r1 = oracle.decode(q, k, v, [6], routing_enabled=False, libpath=lib)
    r2 = oracle.decode(q, k, v, [9], routing_enabled=False, libpath=lib)
    np.testing.assert_array_equal(r1.out, r2.out)


def check_cosine_properties(lib=None):
    D = 8
    rng = np.random.default_rng(11)
    k0 = np.round(rng.standard_normal(D) * 8) / 8
    k0[0] = 1.0
    # an exactly orthogonal vector built from two coordinates
    perp = np.zeros(D)
    perp[0], perp[1] = -k0[1], k0[0]
    qs = np.stack([2.0 * k0, -k0, perp, 0.5 * k0])
    q = bits(qs[None])                                   # [1,4,D]
    k = bits(np.tile(k0, (1, 1, 2, 1)))
    v = bits(np.ones((1, 1, 2, D)))
    r = oracle.route(q, k, [2], tau_coef=(0, 0, 0, 0.0), libpath=lib)      # one group of r = 4
    np.testing.assert_allclose(r.head_cos[0], [1.0, -1.0, 0.0, 1.0], rtol=0, atol=1e-15)
    np.testing.assert_allclose(r.group_score[0, 0], 0.25, rtol=0, atol=1e-15)
    # r = 1: S equals s; |S| <= 1; rescaling q or K_0 by powers of two changes nothing
    q1, k1, _, sl = synth.random_small(500, 2, 4, 4, D, 3)
    a = oracle.route(q1, k1, sl, libpath=lib)
    np.testing.assert_array_equal(a.group_score, a.head_cos)
    assert np.all(np.abs(a.group_score) <= 1.0 + 1e-15)
    q4 = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(q1) * 4.0)
    k4 = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(k1) * 0.5)
    b = oracle.route(q4, k4, sl, libpath=lib)
    np.testing.assert_allclose(b.head_cos, a.head_cos, rtol=0, atol=1e-15)
    # zero query or zero anchor: cosine 0, not NaN
    qz = q1.copy()
    qz[0, 0] = 0
    kz = k1.copy()
    kz[1, 2, 0] = 0
    c = oracle.route(qz, kz, sl, libpath=lib)
    assert c.head_cos[0, 0] == 0.0 and c.head_cos[1, 2] == 0.0 and np.all(np.isfinite(c.head_cos))
    # a supplied anchor norm replaces the recomputed one: doubling it halves the cosine
    kn = np.linalg.norm(f64(k1)[:, :, 0], axis=-1)
    d = oracle.route(q1, k1, sl, k0_norm=kn, libpath=lib)
    np.testing.assert_allclose(d.head_cos, a.head_cos, rtol=1e-14, atol=1e-16)
    e = oracle.route(q1, k1, sl, k0_norm=2 * kn, libpath=lib)
    np.testing.assert_allclose(e.head_cos, a.head_cos / 2, rtol=1e-14, atol=1e-16)


def check_decision_properties(lib=None):
    w = synth.WORKLOADS["c0"].scaled(96)
    sb = synth.generate(w, seed=5)
    args = (sb.q, sb.k, sb.v, sb.seq_lens)
    lo = oracle.decode(*args, tau_coef=(0, 0, 0, -2.0), libpath=lib)
    assert lo.mask.all() and np.all(lo.out == 0.0)
    hi = oracle.decode(*args, tau_coef=(0, 0, 0, 2.0), libpath=lib)
    off = oracle.decode(*args, tau_coef=(0, 0, 0, -2.0), routing_enabled=False, libpath=lib)
    assert not hi.mask.any() and not off.mask.any()
    np.testing.assert_array_equal(hi.out, off.out)
    # skip sets are nested in tau and the count is monotone
    prev = None
    for tau in np.linspace(-1.0, 1.0, 41):
        m = oracle.route(sb.q, sb.k, sb.seq_lens, tau_coef=(0, 0, 0, float(tau)), libpath=lib).mask.astype(bool)
        if prev is not None:
            assert np.all(prev | ~m)       # m subset of prev
        prev = m
    # the mask reads token 0 of K only: scrambling V and every later key row changes nothing
    base = oracle.decode(*args, libpath=lib)
    k2, v2 = sb.k.copy(), sb.v.copy()
    rng = np.random.default_rng(9)
    k2[:, :, 1:] = rng.integers(0, 0x4000, size=k2[:, :, 1:].shape, dtype=np.uint16)
    v2[:] = rng.integers(0, 0x4000, size=v2.shape, dtype=np.uint16)
    alt = oracle.decode(sb.q, k2, v2, sb.seq_lens, libpath=lib)
    np.testing.assert_array_equal(alt.mask, base.mask)
    np.testing.assert_array_equal(alt.group_score, base.group_score)
    assert base.mask.any() and not base.mask.all()
    # a group is all-zero or untouched: rows of one group share the decision
    G = w.group_size
    rows_zero = np.all(base.out == 0.0, axis=-1).reshape(w.batch, w.n_kv_heads, G)
    assert np.array_equal(rows_zero.all(-1), base.mask.astype(bool))
    assert np.array_equal(rows_zero.any(-1), base.mask.astype(bool))
    # per-sequence tau from per-sequence length (x = L/len_norm): only the longer sequence crosses
    q, k, v, sl = synth.random_small(600, 2, 2, 1, 8, 10, [4, 10])
    kf = synth.bf16_bits_to_f32(k)
    qn = synth.f32_to_bf16_bits(np.stack([np.stack([kf[b, 0, 0], kf[b, 0, 0]]) for b in range(2)]))
    r = oracle.decode(qn, k, v, sl, tau_coef=(0, 0, -1.0, 1.5), len_norm=10.0, libpath=lib)
    np.testing.assert_allclose(r.tau, [1.1, 0.5], rtol=0, atol=1e-15)
    assert r.mask[:, 0].tolist() == [0, 1]


def check_skip_error_bound(lib=None):
    """Eq. 3-5: ||u|| <= alpha_0 ||v_0|| + (1 - alpha_0) max_{t>=1} ||v_t||; a skipped head's
    error is exactly ||u||."""
    for name, L in (("c0", 200), ("c2", 333), ("c4", 1500)):
        w = synth.WORKLOADS[name].scaled(L, batch=1)
        sb = synth.generate(w, seed=w.base_seed + 1)
        r = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True, libpath=lib)
        vf = f64(sb.v)
        G = w.group_size
        for b in range(w.batch):
            for h in range(w.n_q_heads):
                g = h // G
                Lb = int(sb.seq_lens[b])
                v0 = np.linalg.norm(vf[b, g, 0])
                vmax = np.linalg.norm(vf[b, g, 1:Lb], axis=-1).max()
                a0 = r.alpha0[b, h]
                un = np.linalg.norm(r.dense_out[b, h])
                assert un <= a0 * v0 + (1 - a0) * vmax + 1e-12
                if r.mask[b, g]:
                    assert np.linalg.norm(r.dense_out[b, h] - r.out[b, h]) == un
        # planted sink heads really are in the target regime (alpha_0 > 0.9 > gamma = 0.65)
        assert np.all(r.alpha0[sb.sink_head] > 0.9)
        assert np.all(r.alpha0[~sb.sink_head] < 0.1)


def check_symmetries(lib=None):
    B, Hq, Hkv, D, L = 1, 6, 2, 8, 21
    q, k, v, sl = synth.random_small(700, B, Hq, Hkv, D, L)
    tau = (0, 0, 0, 0.05)
    base = oracle.decode(q, k, v, sl, tau_coef=tau, want_dense=True, libpath=lib)
    # joint permutation of tokens 1..L-1 of K and V
    perm = np.concatenate([[0], 1 + np.random.default_rng(1).permutation(L - 1)])
    p = oracle.decode(q, k[:, :, perm], v[:, :, perm], sl, tau_coef=tau, want_dense=True, libpath=lib)
    np.testing.assert_allclose(p.dense_out, base.dense_out, rtol=1e-12, atol=1e-14)
    np.testing.assert_array_equal(p.mask, base.mask)
    # permuting the heads inside a group permutes outputs, keeps the mask
    r_ = Hq // Hkv
    hp = np.array([2, 0, 1, 4, 5, 3])
    ph = oracle.decode(q[:, hp], k, v, sl, tau_coef=tau, want_dense=True, libpath=lib)
    np.testing.assert_allclose(ph.dense_out, base.dense_out[:, hp], rtol=0, atol=0)
    np.testing.assert_array_equal(ph.mask, base.mask)
    np.testing.assert_allclose(ph.group_score, base.group_score, rtol=1e-14)
    # groups are independent: changing group 1's data leaves group 0's rows alone
    k2, v2, q2 = k.copy(), v.copy(), q.copy()
    k2[:, 1] = k[:, 1][:, ::-1]
    v2[:, 1] = v[:, 1][:, ::-1]
    q2[:, r_:] = q[:, r_:][:, ::-1]
    alt = oracle.decode(q2, k2, v2, sl, tau_coef=tau, want_dense=True, libpath=lib)
    np.testing.assert_array_equal(alt.dense_out[:, :r_], base.dense_out[:, :r_])
    assert alt.mask[0, 0] == base.mask[0, 0]
    assert not np.allclose(alt.dense_out[:, r_:], base.dense_out[:, r_:])
    # swapping K and V roles is not a symmetry: catches transposed operands
    sw = oracle.decode(q, v, k, sl, routing_enabled=False, libpath=lib)
    assert not np.allclose(sw.out, base.dense_out)


def check_separate_anchor(lib=None):
    """Anchors kept apart from the cache (the K_0 tensor of Section 4.3) drive routing only."""
    B, Hq, Hkv, D, L = 2, 8, 4, 8, 11
    q, k, v, sl = synth.random_small(800, B, Hq, Hkv, D, L, [L, 7])
    tau = (0, 0, 0, 0.0)
    base = oracle.decode(q, k, v, sl, tau_coef=tau, want_dense=True, libpath=lib)
    same = oracle.decode(q, k, v, sl, tau_coef=tau, want_dense=True, k0=k[:, :, 0].copy(), libpath=lib)
    np.testing.assert_array_equal(same.group_score, base.group_score)
    np.testing.assert_array_equal(same.out, base.out)
    # other anchors: routing as if they were row 0, attention still over the real cache
    rng = np.random.default_rng(5)
    k0 = synth.f32_to_bf16_bits(rng.standard_normal((B, Hkv, D)).astype(np.float32))
    alt = oracle.decode(q, k, v, sl, tau_coef=tau, want_dense=True, k0=k0, libpath=lib)
    k_swapped = k.copy()
    k_swapped[:, :, 0] = k0
    ref_route = oracle.route(q, k_swapped, sl, tau_coef=tau, libpath=lib)
    np.testing.assert_array_equal(alt.group_score, ref_route.group_score)
    np.testing.assert_array_equal(alt.mask, ref_route.mask)
    assert not np.array_equal(alt.group_score, base.group_score)
    assert len({tuple(x) for x in alt.group_score.reshape(-1, 1).round(12).tolist()}) == B * Hkv   # one anchor per group
    np.testing.assert_array_equal(alt.dense_out, base.dense_out)
    out, _, _ = library_attention(q, k, v, sl)
    keep = np.repeat(1 - alt.mask, Hq // Hkv, axis=1)[..., None]
    np.testing.assert_allclose(alt.out, out * keep, rtol=1e-12, atol=1e-13)
    # same through the Split-K entry and the route-only entry
    o2, m2, _, _ = oracle.decode_splitk(q, k, v, sl, [0, 4, L], tau_coef=tau, k0=k0, libpath=lib)
    np.testing.assert_array_equal(m2, alt.mask)
    np.testing.assert_allclose(o2, alt.out, rtol=1e-12, atol=1e-13)


def check_paged_gather(lib=None):
    """Gathering pages == numpy fancy indexing; a paged decode == the decode on the contiguous cache it
    came from, whatever the physical page order."""
    B, Hq, Hkv, D, L, pt = 3, 4, 2, 8, 23, 4
    q, k, v, sl = synth.random_small(900, B, Hq, Hkv, D, L, [L, 9, 4])
    ref = oracle.decode(q, k, v, sl, tau_coef=(0, 0, 0, 0.05), want_dense=True, libpath=lib)
    for seed in (1, 2):
        kp, tab = synth.to_pages(k, sl, pt, seed)
        vp, tab2 = synth.to_pages(v, sl, pt, seed)
        assert np.array_equal(tab, tab2)
        got = oracle.gather_pages(kp, tab, sl, L, libpath=lib)
        for b in range(B):
            Lb = int(sl[b])
            t = np.arange(Lb)
            expect = kp[tab[b, t // pt], :, t % pt].transpose(1, 0, 2)       # [Hkv, Lb, D]
            assert np.array_equal(got[b, :, :Lb], expect)
            assert np.array_equal(got[b, :, :Lb], k[b, :, :Lb])
            assert np.all(got[b, :, Lb:] == 0)
        r = oracle.decode_paged(q, kp, vp, tab, sl, L, tau_coef=(0, 0, 0, 0.05), want_dense=True, libpath=lib)
        np.testing.assert_array_equal(r.out, ref.out)
        np.testing.assert_array_equal(r.mask, ref.mask)
        np.testing.assert_array_equal(r.group_score, ref.group_score)
    assert ref.mask.any() and not ref.mask.all()


def check_concentration(lib=None):
    """Table 1's statistics (Section 3): weight of token 0, largest and mean weight of the rest."""
    # hand case: q = [1], keys 0, 1, 2, scale ln 2 -> unnormalised weights 1, 2, 4
    q = bits(np.array([[[1.0]]]))
    k = bits(np.array([[[[0.0], [1.0], [2.0]]]]))
    v = bits(np.array([[[[8.0], [1.0], [-2.0]]]]))
    a0, mx, mean, rest = oracle.concentration(q, k, v, [3], sm_scale=float(np.log(2.0)), libpath=lib)
    np.testing.assert_allclose([a0[0, 0], mx[0, 0], mean[0, 0]], [1 / 7, 4 / 7, 3 / 7], rtol=1e-14)
    np.testing.assert_allclose(rest[0, 0, 0], (2 * 1.0 + 4 * -2.0) / 6, rtol=1e-14)
    # the largest weight may sit on token 0: it must not be reported as the largest of the rest
    k2 = bits(np.array([[[[3.0], [1.0], [2.0]]]]))
    a0, mx, mean, _ = oracle.concentration(q, k2, v, [3], sm_scale=float(np.log(2.0)), libpath=lib)
    np.testing.assert_allclose([a0[0, 0], mx[0, 0], mean[0, 0]], [8 / 14, 4 / 14, 3 / 14], rtol=1e-14)
    # library softmax on grouped heads with ragged lengths; token 0 dropped for out_rest
    B, Hq, Hkv, D, Lmax = 3, 6, 2, 8, 19
    sl = [19, 7, 2]
    qq, kk, vv, _ = synth.random_small(900, B, Hq, Hkv, D, Lmax, sl)
    a0, mx, mean, rest = oracle.concentration(qq, kk, vv, sl, libpath=lib)
    qf = f64(qq)
    kf = np.repeat(f64(kk), Hq // Hkv, axis=1)
    for b in range(B):
        L = sl[b]
        p = softmax(np.einsum("hd,htd->ht", qf[b], kf[b, :, :L]) / np.sqrt(D), axis=-1)
        np.testing.assert_allclose(a0[b], p[:, 0], rtol=1e-12)
        np.testing.assert_allclose(mx[b], p[:, 1:].max(axis=-1), rtol=1e-12)
        np.testing.assert_allclose(mean[b], p[:, 1:].mean(axis=-1), rtol=1e-12)
    np.testing.assert_allclose(a0 + mean * (np.asarray(sl)[:, None] - 1), 1.0, rtol=1e-13)
    assert np.all(mx >= mean - 1e-15)
    ref, _, _ = library_attention(qq, kk[:, :, 1:], vv[:, :, 1:], np.asarray(sl) - 1)
    np.testing.assert_allclose(rest, ref, rtol=1e-11, atol=1e-13)
    # identical keys: every weight is 1/L
    k_same = np.repeat(kk[:, :, :1], Lmax, axis=2)
    a0, mx, mean, _ = oracle.concentration(qq, k_same, vv, sl, libpath=lib)
    for b in range(B):
        np.testing.assert_allclose(a0[b], 1.0 / sl[b], rtol=1e-13)
        np.testing.assert_allclose(mx[b], 1.0 / sl[b], rtol=1e-13)
        np.testing.assert_allclose(mean[b], 1.0 / sl[b], rtol=1e-13)
    # one token: all the weight on it, nothing else; none: undefined
    a0, mx, mean, rest = oracle.concentration(qq, kk, vv, [1, 0, 1], libpath=lib)
    assert np.all(a0[0] == 1.0) and np.all(mx[0] == 0.0) and np.all(mean[0] == 0.0) and np.all(rest[0] == 0.0)
    assert np.all(np.isnan(a0[1])) and np.all(np.isnan(mx[1])) and np.all(np.isnan(mean[1])) and np.all(rest[1] == 0.0)


def check_length_clamp(lib=None):
    """Lengths outside [0, L_max] are clamped before anything uses them: a negative length behaves as 0
    (zero output, mask 0, lse -inf, tau evaluated at x = 0), one beyond the stride as the stride.  The
    threshold is length-dependent here, so a clamp applied to the attention but not to tau shows."""
    B, Hq, Hkv, D, L = 4, 4, 2, 8, 6
    q, k, v, _ = synth.random_small(1000, B, Hq, Hkv, D, L)
    qf, kf = synth.bf16_bits_to_f32(q), synth.bf16_bits_to_f32(k)
    for b in range(B):                       # group 0 of every sequence points along its anchor: S = 1
        qf[b, :2] = kf[b, 0, 0]
    q = synth.f32_to_bf16_bits(qf)
    coef, norm = (0.0, 0.0, 0.25, 0.5), 6.0          # tau(x) = 0.25 x + 0.5, x = L / 6
    sl = [-3, 0, L + 9, L]
    r = oracle.decode(q, k, v, sl, tau_coef=coef, len_norm=norm, want_dense=True, libpath=lib)
    np.testing.assert_allclose(r.tau, [0.5, 0.5, 0.75, 0.75], rtol=0, atol=1e-15)
    for b in (0, 1):                         # no valid row: nothing to attend over, never a Sink Group
        assert np.all(r.out[b] == 0.0) and np.all(r.dense_out[b] == 0.0)
        assert r.mask[b].tolist() == [0, 0]
        assert np.all(np.isneginf(r.lse[b]))
    ref, lse, _ = library_attention(q, k, v, [0, 0, L, L])
    assert r.mask[2].tolist() == [1, 0] and r.mask[3].tolist() == [1, 0]
    np.testing.assert_allclose(r.dense_out, ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(r.lse[2:], lse[2:], rtol=1e-12, atol=1e-13)
    assert np.all(r.out[2:, :2] == 0.0)
    np.testing.assert_allclose(r.out[2:, 2:], ref[2:, 2:], rtol=1e-12, atol=1e-13)
    # the same through the route-only and the Split-K entries
    rr = oracle.route(q, k, sl, tau_coef=coef, len_norm=norm, libpath=lib)
    np.testing.assert_allclose(rr.tau, [0.5, 0.5, 0.75, 0.75], rtol=0, atol=1e-15)
    np.testing.assert_array_equal(rr.mask, r.mask)
    o2, m2, pm, pl = oracle.decode_splitk(q, k, v, sl, [0, 4, L + 20], tau_coef=coef, len_norm=norm, libpath=lib)
    np.testing.assert_array_equal(m2, r.mask)
    np.testing.assert_allclose(o2, r.out, rtol=1e-12, atol=1e-13)
    assert np.all(np.isneginf(pm[:2])) and np.all(pl[:2] == 0.0)
    # concentration statistics and the page gather clamp the same way
    a0, mx, mean, rest = oracle.concentration(q, k, v, sl, libpath=lib)
    assert np.all(np.isnan(a0[:2])) and np.all(rest[:2] == 0.0)
    np.testing.assert_array_equal(a0[2], oracle.concentration(q[2:3], k[2:3], v[2:3], [L], libpath=lib)[0][0])
    kp, tab = synth.to_pages(k, [0, 0, L, L], 2, seed=3)
    got = oracle.gather_pages(kp, tab, sl, L, libpath=lib)
    assert np.all(got[:2] == 0) and np.array_equal(got[2:], k[2:])


def check_nan_norms(lib=None):
    """A cosine whose denominator is not a positive number is 0 (zero or NaN norm alike): a NaN in a
    query, or in the anchor when its norm is recomputed, makes that head's cosine exactly 0, and the
    group mean is the mean of the remaining cosines.  With a finite cached norm and a NaN anchor the
    denominator is fine, the dot product is NaN, the score is NaN, and the strict comparison keeps the
    group active whatever the threshold."""
    D = 8
    k0 = np.array([1.0, 0, 0, 0, 0, 0, 0, 0])
    qs = np.stack([3.0 * k0, 0.5 * k0, -2.0 * k0, k0])              # cosines 1, 1, -1, 1
    q = bits(qs[None])                                               # one group of r = 4, and ...
    q = np.concatenate([q, q], axis=1)                               # ... a second group with the same heads
    k = bits(np.tile(k0, (1, 2, 3, 1)))
    v = bits(np.ones((1, 2, 3, D)))
    base = oracle.decode(q, k, v, [3], tau_coef=(0, 0, 0, 0.4), want_dense=True, libpath=lib)
    np.testing.assert_array_equal(base.head_cos[0], [1, 1, -1, 1, 1, 1, -1, 1])
    np.testing.assert_array_equal(base.group_score[0], [0.5, 0.5])
    assert base.mask[0].tolist() == [1, 1]
    nan = np.uint16(0x7FC0)
    qn = q.copy()
    qn[0, 1, 5] = nan                                                # NaN in one query of group 0
    r = oracle.decode(qn, k, v, [3], tau_coef=(0, 0, 0, 0.4), want_dense=True, libpath=lib)
    assert r.head_cos[0, 1] == 0.0 and not np.signbit(r.head_cos[0, 1])
    np.testing.assert_array_equal(r.head_cos[0], [1, 0, -1, 1, 1, 1, -1, 1])
    np.testing.assert_array_equal(r.group_score[0], [0.25, 0.5])
    assert r.mask[0].tolist() == [0, 1]                              # 0.25 < 0.4 < 0.5
    kn = k.copy()
    kn[0, 1, 0, 2] = nan                                             # NaN in the anchor of group 1, norm recomputed
    r = oracle.decode(q, kn, v, [3], tau_coef=(0, 0, 0, -0.5), want_dense=True, libpath=lib)
    np.testing.assert_array_equal(r.head_cos[0], [1, 1, -1, 1, 0, 0, 0, 0])
    np.testing.assert_array_equal(r.group_score[0], [0.5, 0.0])
    assert r.mask[0].tolist() == [1, 1]                              # S = 0 > -0.5: the zero cosines do count
    r = oracle.route(q, kn, [3], tau_coef=(0, 0, 0, 0.0), libpath=lib)
    assert r.mask[0].tolist() == [1, 0]                              # 0 > 0 is false
    # the same anchor kept apart from the cache
    r = oracle.route(q, k, [3], tau_coef=(0, 0, 0, -0.5), k0=kn[:, :, 0].copy(), libpath=lib)
    np.testing.assert_array_equal(r.group_score[0], [0.5, 0.0])
    # finite cached norm, NaN anchor: NaN score, group active even at tau = -2
    r = oracle.route(q, kn, [3], tau_coef=(0, 0, 0, -2.0), k0_norm=np.ones((1, 2)), libpath=lib)
    assert np.isnan(r.group_score[0, 1]) and r.group_score[0, 0] == 0.5
    assert r.mask[0].tolist() == [1, 0]
    # a cached norm that is negative or NaN counts as "not cached": the norm is recomputed from the anchor
    for bad in (np.nan, -1.0):
        r = oracle.route(q, k, [3], tau_coef=(0, 0, 0, 0.4), k0_norm=np.array([[2.0, bad]]), libpath=lib)
        np.testing.assert_array_equal(r.group_score[0], [0.25, 0.5])
        assert r.mask[0].tolist() == [0, 1]


ALL_PINS = [check_golden, check_brute_force_dense, check_routed_vs_library,
            check_splitk_equals_single_pass, check_closed_forms, check_cosine_properties,
            check_decision_properties, check_skip_error_bound, check_symmetries, check_separate_anchor, check_paged_gather,
            check_concentration, check_length_clamp, check_nan_norms]
