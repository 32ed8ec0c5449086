"""Paged KV cache: HIP path vs the oracle's gather-then-decode, and vs the contiguous HIP path (needs an MI355X)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2604_16883_amd import binding, synth

import gpu_util as gu


def run_paged(sb, kp, vp, table, page_tokens, given_lens=None, **kw):
    import torch
    w = sb.workload
    B, Hq, Hkv = w.batch, w.n_q_heads, w.n_kv_heads
    Lmax = sb.max_seq_len
    dev = dict(q=gu.to_dev(sb.q), k=gu.to_dev(kp), v=gu.to_dev(vp), sl=gu.to_dev(np.asarray(sb.seq_lens if given_lens is None else given_lens, np.int32)),
               t=gu.to_dev(table))
    p = binding.make_route_params(B, Hq, Hkv, Lmax, **kw)
    plan = binding.sinkrouter_plan(p)
    ws = torch.empty((plan.workspace_bytes,), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    p.workspace, p.workspace_bytes = ws.data_ptr(), plan.workspace_bytes
    lay = binding.make_paged_layout(page_tokens, table.shape[1], kp.shape[0])
    out = torch.full((B, Hq, 128), -1, dtype=torch.int16, device="cuda")
    mask = torch.full((B, Hkv), 7, dtype=torch.uint8, device="cuda")
    binding.sinkrouter_decode_paged(dev["q"], dev["k"], dev["v"], dev["t"], dev["sl"], p, lay, out, mask)
    torch.cuda.synchronize()
    bits = out.cpu().numpy().view(np.uint16)
    return dict(out=synth.bf16_bits_to_f32(bits), out_bits=bits, mask=mask.cpu().numpy(), plan=plan)


CASES = [("c0", 1733, None, 64), ("c1", 1000, [1000, 937, 64, 1], 128), ("c2", 3125, None, 256),
         ("c4", 1500, [1500, 0], 64), ("c3", 2049, None, 1024)]


@pytest.mark.parametrize("name,L,sl,pt", CASES, ids=["%s-p%d" % (c[0], c[3]) for c in CASES])
def test_paged_matches_oracle_and_contiguous(name, L, sl, pt):
    w = synth.WORKLOADS[name].scaled(L)
    sb = synth.generate(w, seq_lens=sl)
    kp, table = synth.to_pages(sb.k, sb.seq_lens, pt, seed=11)
    vp, _ = synth.to_pages(sb.v, sb.seq_lens, pt, seed=11)
    for kw in (dict(), dict(routing_enabled=False), dict(num_splits=5)):
        res = run_paged(sb, kp, vp, table, pt, **kw)
        ref = oracle.decode_paged(sb.q, kp, vp, table, sb.seq_lens, sb.max_seq_len, want_dense=True,
                                  routing_enabled=kw.get("routing_enabled", True))
        cont = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, **kw)
        res["probe_mask"], res["score"] = cont["probe_mask"], cont["score"]
        rep = gu.compare(res, ref, w.group_size, "%s paged %s" % (name, kw))
        # same schedule, same arithmetic: the paged result equals the contiguous one bit for bit
        assert np.array_equal(res["out_bits"], cont["out_bits"]) and np.array_equal(res["mask"], cont["mask"])
        print(name, "paged", pt, kw, rep, flush=True)


def test_paged_full_size_c1():
    w = synth.WORKLOADS["c1"]
    sb = synth.generate(w)
    kp, table = synth.to_pages(sb.k, sb.seq_lens, 256, seed=3)
    vp, _ = synth.to_pages(sb.v, sb.seq_lens, 256, seed=3)
    res = run_paged(sb, kp, vp, table, 256)
    ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True)
    cont = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens)
    res["probe_mask"], res["score"] = cont["probe_mask"], cont["score"]
    print("c1 paged full", gu.compare(res, ref, w.group_size, "c1 paged full"), flush=True)
    assert np.array_equal(res["out_bits"], cont["out_bits"])


def test_full_size_ragged_batch_contiguous_and_paged():
    """A 128K-class batch with one long and several short sequences (32768, 20011, 4097 and 65 tokens, the
    shape the benchmark times as c1_ragged): the balanced schedule deals the long sequence's blocks over most
    workgroups while the short ones share a few, tails fall inside a block and inside a page.  Contiguous and
    paged (256-token pages, random page order), routed at three thresholds and dense, element by element
    against the oracle; the paged result equals the contiguous one bit for bit."""
    lens = [32768, 20011, 4097, 65]
    w = synth.WORKLOADS["c1"].scaled(max(lens), batch=len(lens))
    sb = synth.generate(w, seq_lens=lens)
    kp, table = synth.to_pages(sb.k, sb.seq_lens, 256, seed=17)
    vp, _ = synth.to_pages(sb.v, sb.seq_lens, 256, seed=17)
    dev = None
    seen = set()
    for kw in (dict(tau_coef=(0, 0, 0, 0.55)), dict(tau_coef=(0, 0, 0, 0.45)), dict(tau_coef=(0, 0, 0, 0.7)), dict(routing_enabled=False)):
        print("ragged full", kw, flush=True)
        ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True, **kw)
        cont = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, dev=dev, **kw)
        dev = cont["dev"]
        rep = gu.compare(cont, ref, w.group_size, "ragged full %s" % kw)
        assert cont["plan"].schedule == 1
        res = run_paged(sb, kp, vp, table, 256, **kw)
        assert np.array_equal(res["out_bits"], cont["out_bits"]) and np.array_equal(res["mask"], cont["mask"])
        seen.add(rep["skip_ratio"])
        print("ragged full", kw, rep, flush=True)
    assert len(seen) >= 3
