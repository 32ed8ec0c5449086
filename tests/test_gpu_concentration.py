"""GPU parity of the attention-concentration statistics (Section 3, Table 1) against the CPU oracle
(needs an MI355X)."""
import dataclasses

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2604_16883_amd import analysis, binding, synth

import gpu_util as gu


def _run(sb, **kw):
    import torch
    w = sb.workload
    B, Hq, Hkv, Lmax = w.batch, w.n_q_heads, w.n_kv_heads, sb.max_seq_len
    dev = dict(q=gu.to_dev(sb.q), k=gu.to_dev(sb.k), v=gu.to_dev(sb.v), sl=gu.to_dev(sb.seq_lens))
    p = binding.make_route_params(B, Hq, Hkv, Lmax, **kw)
    plan = binding.sinkrouter_plan(p)
    ws = torch.empty((plan.workspace_bytes,), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    p.workspace, p.workspace_bytes = ws.data_ptr(), plan.workspace_bytes
    out = torch.full((B, Hq, 128), -1, dtype=torch.int16, device="cuda")
    mask = torch.full((B, Hkv), 7, dtype=torch.uint8, device="cuda")
    st = [torch.full((B, Hq), 123.0, dtype=torch.float32, device="cuda") for _ in range(3)]
    binding.sinkrouter_concentration(dev["q"], dev["k"], dev["v"], dev["sl"], p, out, mask, *st)
    torch.cuda.synchronize()
    assert not mask.cpu().numpy().any()                     # routing plays no part
    rest = synth.bf16_bits_to_f32(out.cpu().numpy().view(np.uint16)).astype(np.float64)
    return [t.cpu().numpy().astype(np.float64) for t in st] + [rest]


def _check(sb, got, label):
    a0, mx, mean, rest = got
    ra0, rmx, rmean, rrest = oracle.concentration(sb.q, sb.k, sb.v, sb.seq_lens)
    Hq = sb.workload.n_q_heads
    lens = np.repeat(np.asarray(sb.seq_lens), Hq).reshape(len(sb.seq_lens), Hq)
    live = lens > 0
    np.testing.assert_allclose(a0[live], ra0[live], rtol=3e-4, atol=1e-7, err_msg=label)
    np.testing.assert_allclose(mx[live], rmx[live], rtol=3e-4, atol=1e-12, err_msg=label)
    np.testing.assert_allclose(mean[live], rmean[live], rtol=3e-4, atol=1e-12, err_msg=label)
    for t in (a0, mx, mean):
        assert np.all(np.isnan(t[~live])), label
    one = lens == 1
    assert np.all(a0[one] == 1.0) and np.all(mx[one] == 0.0) and np.all(mean[one] == 0.0), label
    err = np.abs(rest - rrest)
    assert float(err.max()) <= gu.MAX_ABS_TOL, (label, float(err.max()))
    den = np.sqrt((rrest ** 2).sum(-1))
    num = np.sqrt((err ** 2).sum(-1))
    assert np.all(num[den > 0] / den[den > 0] <= gu.REL_L2_TOL), label
    assert np.all(rest[lens <= 1] == 0.0), label
    print(label, "concentration parity ok; max rel d(max_rest)",
          float(np.max(np.abs(mx[live] - rmx[live]) / np.maximum(rmx[live], 1e-300))), flush=True)
    return ra0, rmx, rmean


@pytest.mark.parametrize("name,L,sl,splits", [("c0", 1500, None, 0), ("c2", 3125, None, 0), ("c4", 900, [900, 0], 0),
                                              ("c1", 700, [700, 1, 65, 2], 0), ("c0", 1500, None, 3),
                                              ("c4", 321, [1, 321], 2)])
def test_concentration_matches_oracle(name, L, sl, splits):
    w = synth.WORKLOADS[name].scaled(L)
    sb = synth.generate(w, seq_lens=sl)
    _check(sb, _run(sb, num_splits=splits), "%s L%d splits%d" % (name, L, splits))


def test_concentration_ignores_routing_fields_and_leaves_decode_unchanged():
    """Routing switches and cached anchors of the parameter block play no part, and a decode call
    on the same workspace afterwards is unaffected."""
    import torch
    w = synth.WORKLOADS["c0"].scaled(1000)
    sb = synth.generate(w)
    base = _run(sb)
    junk = torch.full((w.batch, w.n_kv_heads), 3.0, dtype=torch.float32, device="cuda")
    other = _run(sb, routing_enabled=True, tau_coef=(0, 0, 0, -2.0), k0_norm=junk)
    for x, y in zip(base, other):
        np.testing.assert_array_equal(x, y)
    res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens)
    gu.compare(res, oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True), w.group_size, "after concentration")


def test_table_of_regimes_from_graded_sink_gains():
    """Heads with graded pull toward token 0 fill the table's regimes; the GPU's table equals the
    oracle's and shows the table's qualitative fact: the more weight on token 0, the larger its ratio
    to the strongest other token."""
    cols_gpu, cols_ref = [], []
    for i, gain in enumerate((9.0, 11.0, 13.0, 15.0, 17.0)):
        w = dataclasses.replace(synth.WORKLOADS["c0"].scaled(2000), sink_gain=gain, sink_frac=1.0, planted_per_head=0)
        sb = synth.generate(w, seed=50 + i)
        got = _run(sb)
        ref = _check(sb, got, "gain %g" % gain)
        cols_gpu.append([x.ravel() for x in got[:3]])
        cols_ref.append([x.ravel() for x in ref])
    g = [np.concatenate([c[j] for c in cols_gpu]) for j in range(3)]
    r = [np.concatenate([c[j] for c in cols_ref]) for j in range(3)]
    # heads whose alpha_0 sits on a bin edge could fall on either side in fp32: left out on both sides
    edge = np.zeros(r[0].shape, bool)
    for regime in (0.4, 0.6, 0.8):
        edge |= np.abs(np.abs(r[0] - regime) - 0.1) < 1e-3
    g = [x[~edge] for x in g]
    r = [x[~edge] for x in r]
    tg = analysis.concentration_table(*g, half_width=0.1)
    tr = analysis.concentration_table(*r, half_width=0.1)
    filled = [k for k in tr if tr[k]["heads"] > 0]
    assert len(filled) >= 2, tr
    for k in filled:
        assert tg[k]["heads"] == tr[k]["heads"]
        for f in ("bos", "max", "mean", "ratio"):
            assert abs(tg[k][f] - tr[k][f]) <= 1e-3 * abs(tr[k][f]), (k, f, tg[k], tr[k])
    ratios = [tr[k]["ratio"] for k in sorted(filled)]
    assert all(a < b for a, b in zip(ratios, ratios[1:])), tr
    print("regime table", tg, flush=True)
