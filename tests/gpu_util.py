"""Helpers for the GPU parity tests: run the HIP path through the C ABI binding and compare
with the CPU oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2604_16883_amd import binding, synth

MAX_ABS_TOL = 1e-2       # stated tolerance: bf16 inputs, fp32 accumulation, bf16 output
REL_L2_TOL = 5e-3
BAND = 1e-4              # routing decisions this close to the threshold are exempt, and counted


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16) if a.dtype == np.uint16 else np.ascontiguousarray(a)).cuda()


def run_hip(q, k, v, seq_lens, *, tau_coef=(0, 0, 0, 0.55), len_norm=0.0, sm_scale=0.0,
            routing_enabled=True, num_splits=0, k0_norm=None, dev=None, profiled=False, k0=None, k0_norm_dev=None):
    """One decode step on the GPU. Returns dict(out fp32 [B,Hq,D], mask uint8 [B,Hkv], score fp32, plan)."""
    import torch
    B, Hq, D = q.shape
    Hkv, Lmax = k.shape[1], k.shape[2]
    if dev is None:
        dev = dict(q=to_dev(q), k=to_dev(k), v=to_dev(v), sl=to_dev(np.asarray(seq_lens, np.int32)))
    kn = k0_norm_dev if k0_norm is None else to_dev(np.asarray(k0_norm, np.float32))
    p = binding.make_route_params(B, Hq, Hkv, Lmax, head_dim=D, num_splits=num_splits,
                                  routing_enabled=routing_enabled, sm_scale=sm_scale,
                                  tau_coef=tau_coef, len_norm=len_norm, k0_norm=kn, k0=k0)
    plan = binding.sinkrouter_plan(p)
    ws = torch.empty((plan.workspace_bytes,), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)      # NaN pattern: an unwritten partial slot that gets read shows up
    p.workspace = ws.data_ptr()
    p.workspace_bytes = plan.workspace_bytes
    out = torch.full((B, Hq, D), -1, dtype=torch.int16, device="cuda")     # 0xFFFF = NaN
    mask = torch.full((B, Hkv), 7, dtype=torch.uint8, device="cuda")
    score = torch.full((B, Hkv), float("nan"), dtype=torch.float32, device="cuda")
    stage = None
    if profiled:
        stage = binding.sinkrouter_decode_profiled(dev["q"], dev["k"], dev["v"], dev["sl"], p, out, mask)
    else:
        binding.sinkrouter_decode(dev["q"], dev["k"], dev["v"], dev["sl"], p, out, mask)
    mask2 = torch.full((B, Hkv), 9, dtype=torch.uint8, device="cuda")
    binding.sinkrouter_probe(dev["q"], dev["k"], dev["sl"], p, score, mask2)
    torch.cuda.synchronize()
    out_bits = out.cpu().numpy().view(np.uint16)
    res = dict(out=synth.bf16_bits_to_f32(out_bits), out_bits=out_bits, mask=mask.cpu().numpy(),
               probe_mask=mask2.cpu().numpy(), score=score.cpu().numpy(), plan=plan, stage_us=stage, dev=dev)
    return res


def compare(res, ref: oracle.OracleResult, group_size: int, label: str = ""):
    """Asserts the stated parity bar; returns a small report."""
    mask, omask = res["mask"], ref.mask
    assert np.array_equal(mask, res["probe_mask"]), label + ": decode and probe disagree on the mask"
    near = np.abs(ref.group_score - ref.tau[:, None]) <= BAND
    disagree = mask != omask
    assert not np.any(disagree & ~near), "%s: skip mask differs outside the %g band at %s" % (
        label, BAND, np.argwhere(disagree & ~near).tolist())
    # S_g itself: fp32 on the GPU
    np.testing.assert_allclose(res["score"], ref.group_score, rtol=0, atol=2e-5, err_msg=label)
    out = res["out"].astype(np.float64)
    # expected output under the GPU's own decision inside the band (dense_out is available there)
    exp = ref.out.copy()
    if np.any(disagree):
        assert ref.dense_out is not None
        for b, g in np.argwhere(disagree):
            rows = slice(g * group_size, (g + 1) * group_size)
            exp[b, rows] = 0.0 if mask[b, g] else ref.dense_out[b, rows]
    assert np.all(np.isfinite(out)), label + ": non-finite output"
    skipped_rows = np.repeat(mask.astype(bool), group_size, axis=1)
    assert np.all(res["out_bits"][skipped_rows] == 0), label + ": Sink Group rows must be exact zeros"
    err = np.abs(out - exp)
    max_abs = float(err.max()) if err.size else 0.0
    num = np.sqrt((err ** 2).sum(-1))
    den = np.sqrt((exp ** 2).sum(-1))
    active = den > 0
    rel_rows = num[active] / den[active]
    rel_l2 = float(np.sqrt((err ** 2).sum()) / max(np.sqrt((exp ** 2).sum()), 1e-300)) if active.any() else 0.0
    worst_row = float(rel_rows.max()) if rel_rows.size else 0.0
    assert max_abs <= MAX_ABS_TOL, "%s: max-abs %g" % (label, max_abs)
    assert rel_l2 <= REL_L2_TOL, "%s: rel-L2 %g" % (label, rel_l2)
    assert worst_row <= 2 * REL_L2_TOL, "%s: worst per-head rel-L2 %g" % (label, worst_row)
    return dict(max_abs=max_abs, rel_l2=rel_l2, worst_row_rel_l2=worst_row, near_threshold=int(near.sum()),
                mask_disagree_in_band=int(disagree.sum()), skip_ratio=float(mask.mean()))
