"""The allocation-free entry point (sinkrouter_decode_static) against sinkrouter_decode, through the C ABI
(needs an MI355X).  Same kernels and schedule on a different buffer, so the results must agree bit for
bit; the parity bar against the oracle is checked on top.  Two calls in a row share the library's static
scratch, the second with a smaller input, so stale records of the first call lie behind the second's."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2604_16883_amd import binding, synth

import gpu_util as gu


def run_static(sb, **kw):
    import torch
    w = sb.workload
    B, Hq, Hkv, Lmax = w.batch, w.n_q_heads, w.n_kv_heads, sb.max_seq_len
    dev = dict(q=gu.to_dev(sb.q), k=gu.to_dev(sb.k), v=gu.to_dev(sb.v), sl=gu.to_dev(sb.seq_lens))
    p = binding.make_route_params(B, Hq, Hkv, Lmax, **kw)          # no workspace
    out = torch.full((B, Hq, 128), -1, dtype=torch.int16, device="cuda")
    mask = torch.full((B, Hkv), 7, dtype=torch.uint8, device="cuda")
    binding.sinkrouter_decode_static(dev["q"], dev["k"], dev["v"], dev["sl"], p, out, mask)
    torch.cuda.synchronize()
    bits = out.cpu().numpy().view(np.uint16)
    return dict(out=synth.bf16_bits_to_f32(bits), out_bits=bits, mask=mask.cpu().numpy())


def test_static_scratch_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    cases = [
        (synth.WORKLOADS["c1"].scaled(3000), [3000, 2933, 64, 1], dict()),               # first call: the larger input
        (synth.WORKLOADS["c0"].scaled(700), None, dict()),                               # then a smaller one
        (synth.WORKLOADS["c2"].scaled(1500), None, dict(num_splits=4)),                  # fixed chunks
        (synth.WORKLOADS["c4"].scaled(900), [900, 0], dict(routing_enabled=False)),      # dense, one empty sequence
    ]
    for w, sl, kw in cases:
        print("static", w.name, sl, kw, flush=True)
        sb = synth.generate(w, seq_lens=sl)
        got = run_static(sb, **kw)
        want = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, **kw)
        assert np.array_equal(got["mask"], want["mask"])
        assert np.array_equal(got["out_bits"], want["out_bits"])
        ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True,
                            routing_enabled=kw.get("routing_enabled", True))
        got["probe_mask"], got["score"] = want["probe_mask"], want["score"]
        print("static", w.name, gu.compare(got, ref, w.group_size, "static " + w.name), flush=True)


def test_static_scratch_rejects_shapes_beyond_its_size():
    p = binding.make_route_params(16, 32, 8, 32768)                 # 512 heads x 257 records: 68 MB
    assert binding.sinkrouter_plan(p).workspace_bytes > binding.STATIC_SCRATCH_BYTES
    rc = binding.sinkrouter_decode_static(1 << 16, 1 << 17, 1 << 18, 1 << 19, p, 1 << 20, 1 << 21, check=False)
    assert rc == binding.SR_ERR_STATIC_LIMIT


def test_static_scratch_call_captured_into_a_graph():
    """The callers this entry point is for: a HIP graph captured around it (after one eager call on the device, which
    looks the scratch array's address up) replays to the eager result every time, with other work between the replays."""
    import torch
    w = synth.WORKLOADS["c1"].scaled(2500, batch=2)
    sb = synth.generate(w, seed=23, seq_lens=[2500, 1301])
    B, Hq, Hkv, Lmax = w.batch, w.n_q_heads, w.n_kv_heads, sb.max_seq_len
    tq, tk, tv, tsl = gu.to_dev(sb.q), gu.to_dev(sb.k), gu.to_dev(sb.v), gu.to_dev(sb.seq_lens)
    p = binding.make_route_params(B, Hq, Hkv, Lmax)
    out = torch.empty((B, Hq, 128), dtype=torch.int16, device="cuda")
    mask = torch.empty((B, Hkv), dtype=torch.uint8, device="cuda")

    def step():
        binding.sinkrouter_decode_static(tq, tk, tv, tsl, p, out, mask)

    step()
    torch.cuda.synchronize()
    eager_out, eager_mask = out.clone(), mask.clone()
    want = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens)
    assert np.array_equal(eager_out.cpu().numpy().view(np.uint16), want["out_bits"])
    assert 0 < int(eager_mask.sum()) < eager_mask.numel()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    other = synth.generate(synth.WORKLOADS["c0"].scaled(900), seed=5)
    for rep in range(4):
        out.fill_(-1)
        mask.fill_(9)
        gu.run_hip(other.q, other.k, other.v, other.seq_lens)        # eager work with its own workspace in between
        run_static(other)                                            # and a call that overwrites the shared scratch
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager_out), "replay %d differs from the eager result" % rep
        assert torch.equal(mask, eager_mask)
