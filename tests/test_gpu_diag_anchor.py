"""GPU parity of the diagnostics (log-sum-exp, alpha_0), the anchor extraction kernel, separately
cached anchors, and calibration on probe scores, against the CPU oracle (needs an MI355X)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2604_16883_amd import analysis, binding, calibrate, synth

import gpu_util as gu


def _run_diag(sb, **kw):
    import torch
    w = sb.workload
    B, Hq, Hkv, Lmax = w.batch, w.n_q_heads, w.n_kv_heads, sb.max_seq_len
    dev = dict(q=gu.to_dev(sb.q), k=gu.to_dev(sb.k), v=gu.to_dev(sb.v), sl=gu.to_dev(sb.seq_lens))
    p = binding.make_route_params(B, Hq, Hkv, Lmax, **kw)
    plan = binding.sinkrouter_plan(p)
    ws = torch.empty((plan.workspace_bytes,), dtype=torch.uint8, device="cuda")
    p.workspace, p.workspace_bytes = ws.data_ptr(), plan.workspace_bytes
    out = torch.full((B, Hq, 128), -1, dtype=torch.int16, device="cuda")
    mask = torch.full((B, Hkv), 7, dtype=torch.uint8, device="cuda")
    lse = torch.full((B, Hq), 123.0, dtype=torch.float32, device="cuda")
    a0 = torch.full((B, Hq), 123.0, dtype=torch.float32, device="cuda")
    binding.sinkrouter_decode_diag(dev["q"], dev["k"], dev["v"], dev["sl"], p, out, mask, lse, a0)
    torch.cuda.synchronize()
    return (synth.bf16_bits_to_f32(out.cpu().numpy().view(np.uint16)), mask.cpu().numpy(), lse.cpu().numpy(), a0.cpu().numpy(), dev)


@pytest.mark.parametrize("name,L,sl", [("c0", 1500, None), ("c2", 3125, None), ("c4", 900, [900, 0])])
def test_lse_and_alpha0_match_oracle(name, L, sl):
    w = synth.WORKLOADS[name].scaled(L)
    sb = synth.generate(w, seq_lens=sl)
    G = w.group_size
    # dense: every head is computed
    out, mask, lse, a0, _ = _run_diag(sb, routing_enabled=False)
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, routing_enabled=False, want_dense=True)
    live = np.repeat(sb.seq_lens > 0, w.n_q_heads).reshape(w.batch, -1)
    np.testing.assert_allclose(lse[live], ref.lse[live], rtol=0, atol=2e-4)
    np.testing.assert_allclose(a0[live], ref.alpha0[live], rtol=2e-4, atol=1e-6)
    assert np.all(np.isneginf(lse[~live])) and np.all(np.isnan(a0[~live]))
    # planted structure shows up in the GPU's own diagnostics
    sink = sb.sink_head & live
    assert np.all(a0[sink] > 0.9) and np.all(a0[~sb.sink_head & live] < 0.1)
    # routed: heads of Sink Groups are not computed (NaN), the rest agree
    out, mask, lse, a0, _ = _run_diag(sb)
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=False)
    assert np.array_equal(mask, ref.mask)
    skipped = np.repeat(mask.astype(bool), G, axis=1)
    assert np.all(np.isnan(lse[skipped])) and np.all(np.isnan(a0[skipped]))
    act = ~skipped & live
    np.testing.assert_allclose(lse[act], ref.lse[act], rtol=0, atol=2e-4)
    np.testing.assert_allclose(a0[act], ref.alpha0[act], rtol=2e-4, atol=1e-6)
    print(name, "lse/alpha0 parity ok; max |dlse|", float(np.abs(lse[act] - ref.lse[act]).max()), flush=True)


def test_extract_anchor_and_separate_anchor_tensor():
    import torch
    w = synth.WORKLOADS["c1"].scaled(700, batch=3)
    sb = synth.generate(w, seed=9, seq_lens=[700, 350, 10])
    B, Hq, Hkv = w.batch, w.n_q_heads, w.n_kv_heads
    dev = dict(q=gu.to_dev(sb.q), k=gu.to_dev(sb.k), v=gu.to_dev(sb.v), sl=gu.to_dev(sb.seq_lens))
    p = binding.make_route_params(B, Hq, Hkv, sb.max_seq_len)
    k0 = torch.full((B, Hkv, 128), -1, dtype=torch.int16, device="cuda")
    kn = torch.full((B, Hkv), -1.0, dtype=torch.float32, device="cuda")
    binding.sinkrouter_extract_anchor(dev["k"], p, k0, kn)
    torch.cuda.synchronize()
    assert np.array_equal(k0.cpu().numpy().view(np.uint16), sb.k[:, :, 0])            # bit-exact copy of row 0
    norm = np.linalg.norm(synth.bf16_bits_to_f32(sb.k[:, :, 0]).astype(np.float64), axis=-1)
    np.testing.assert_allclose(kn.cpu().numpy(), norm, rtol=1e-6)
    # routing from the extracted anchors + cached norms == routing from the cache, bit for bit
    base = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, dev=dev)
    alt = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, dev=dev, k0=k0, k0_norm_dev=kn)
    assert np.array_equal(alt["score"], base["score"]) and np.array_equal(alt["mask"], base["mask"])
    assert np.array_equal(alt["out_bits"], base["out_bits"])
    # anchors that differ from row 0 drive routing only; attention still reads the cache
    rng = np.random.default_rng(3)
    other = synth.f32_to_bf16_bits(rng.standard_normal((B, Hkv, 128)).astype(np.float32))
    for h in range(4):                       # make one group of each sequence sink-like w.r.t. the new anchors
        other[:, 0] = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(sb.q[:, :4]).mean(1))
    res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, dev=dev, k0=gu.to_dev(other), tau_coef=(0, 0, 0, 0.3))
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, k0=other, tau_coef=(0, 0, 0, 0.3), want_dense=True)
    rep = gu.compare(res, ref, w.group_size, "separate anchors")
    assert 0 < rep["skip_ratio"] < 1
    print("separate anchors", rep, flush=True)


def test_calibration_on_probe_scores():
    """Appendix A on synthetic caches: thresholds per length from GPU probe scores, cubic fit, and the
    fitted rule realises the target skip ratio when fed back through the routed decode."""
    by_len, batches = {}, {}
    for L in (512, 1024, 2048, 4096):
        s = []
        for seed in range(3):
            sb = synth.generate(synth.WORKLOADS["c1"].scaled(L), seed=700 + seed)
            dev = dict(q=gu.to_dev(sb.q), k=gu.to_dev(sb.k), sl=gu.to_dev(sb.seq_lens))
            sc = calibrate.probe_scores(dev["q"], dev["k"], dev["sl"])
            np.testing.assert_allclose(sc, oracle.route(sb.q, sb.k, sb.seq_lens).group_score, rtol=0, atol=2e-5)
            s.append(sc.ravel())
            batches[(L, seed)] = sb
        by_len[L] = np.concatenate(s)
    cal = calibrate.calibrate(by_len, target=0.6)
    print("calibration", cal["tau_coef"], cal["realised_skip_ratio"], flush=True)
    skipped = total = 0
    for (L, seed), sb in batches.items():
        res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=cal["tau_coef"], len_norm=cal["len_norm"])
        ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, tau_coef=cal["tau_coef"], len_norm=cal["len_norm"], want_dense=True)
        gu.compare(res, ref, 4, "calibrated L=%d seed=%d" % (L, seed))
        skipped += int(res["mask"].sum())
        total += res["mask"].size
    assert abs(skipped / total - 0.6) <= 0.05


def test_proxy_reliability_from_gpu_outputs():
    """Appendix C's analysis on the library's own outputs: S_g from the probe, alpha_0 from a dense run."""
    scores, a0g = [], []
    for seed in range(4):
        w = synth.WORKLOADS["c1"].scaled(2048)
        sb = synth.generate(w, seed=900 + seed)
        out, mask, lse, a0, dev = _run_diag(sb, routing_enabled=False)
        scores.append(calibrate.probe_scores(dev["q"], dev["k"], dev["sl"]).ravel())
        a0g.append(analysis.group_alpha0(a0, w.group_size).ravel())
    scores, a0g = np.concatenate(scores), np.concatenate(a0g)
    labels = analysis.sink_labels(a0g)
    ap = analysis.average_precision(scores, labels)
    sw = analysis.threshold_sweep(scores, labels, [0.55])
    print("AUPRC", ap, "at tau 0.55:", {k: float(v[0]) for k, v in sw.items()}, flush=True)
    assert ap > 0.9
