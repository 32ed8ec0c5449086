"""The decode step can be captured into a HIP graph (it allocates nothing, records no memset and never
synchronises) and every replay reproduces the eager result (needs an MI355X)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2604_16883_amd import binding, synth

import gpu_util as gu


@pytest.mark.parametrize("paged", [False, True], ids=["contiguous", "paged"])
def test_graph_replays_match_eager(paged):
    import torch
    w = synth.WORKLOADS["c1"].scaled(3000, batch=2)
    sb = synth.generate(w, seed=21, seq_lens=[3000, 1777])
    B, Hq, Hkv, Lmax = w.batch, w.n_q_heads, w.n_kv_heads, sb.max_seq_len
    tq, tsl = gu.to_dev(sb.q), gu.to_dev(sb.seq_lens)
    if paged:
        kp, tab = synth.to_pages(sb.k, sb.seq_lens, 128, seed=1)
        vp, _ = synth.to_pages(sb.v, sb.seq_lens, 128, seed=1)
        tk, tv, tt = gu.to_dev(kp), gu.to_dev(vp), gu.to_dev(tab)
        lay = binding.make_paged_layout(128, tab.shape[1], kp.shape[0])
    else:
        tk, tv = gu.to_dev(sb.k), gu.to_dev(sb.v)
    p = binding.make_route_params(B, Hq, Hkv, Lmax)
    plan = binding.sinkrouter_plan(p)
    ws = torch.empty((plan.workspace_bytes,), dtype=torch.uint8, device="cuda")
    p.workspace, p.workspace_bytes = ws.data_ptr(), plan.workspace_bytes
    out = torch.empty((B, Hq, 128), dtype=torch.int16, device="cuda")
    mask = torch.empty((B, Hkv), dtype=torch.uint8, device="cuda")

    def step():
        if paged:
            binding.sinkrouter_decode_paged(tq, tk, tv, tt, tsl, p, lay, out, mask)
        else:
            binding.sinkrouter_decode(tq, tk, tv, tsl, p, out, mask)

    step()
    torch.cuda.synchronize()
    eager_out, eager_mask = out.clone(), mask.clone()
    assert 0 < int(eager_mask.sum()) < eager_mask.numel()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(4):
        out.fill_(-1)                            # eager work between the replays
        mask.fill_(9)
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager_out), "replay %d differs from the eager result" % rep
        assert torch.equal(mask, eager_mask)
    # the queries change between decode steps while the graph stays the same
    tq.copy_(gu.to_dev(np.roll(sb.q, 1, axis=1)))
    step()
    torch.cuda.synchronize()
    ref_out = out.clone()
    out.fill_(-1)
    g.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out)


def test_concurrent_streams_with_distinct_workspaces():
    """Calls on two streams with their own workspaces and outputs may overlap; each reproduces what
    it gives alone."""
    import torch
    w = synth.WORKLOADS["c1"].scaled(20000, batch=2)
    sbs = [synth.generate(w, seed=31), synth.generate(w, seed=32)]
    B, Hq, Hkv, Lmax = w.batch, w.n_q_heads, w.n_kv_heads, sbs[0].max_seq_len
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ctx = []
    for sb, st in zip(sbs, streams):
        p = binding.make_route_params(B, Hq, Hkv, Lmax, stream=st.cuda_stream)
        plan = binding.sinkrouter_plan(p)
        ws = torch.empty((plan.workspace_bytes,), dtype=torch.uint8, device="cuda")
        p.workspace, p.workspace_bytes = ws.data_ptr(), plan.workspace_bytes
        ctx.append(dict(p=p, ws=ws, q=gu.to_dev(sb.q), k=gu.to_dev(sb.k), v=gu.to_dev(sb.v), sl=gu.to_dev(sb.seq_lens),
                        out=torch.empty((B, Hq, 128), dtype=torch.int16, device="cuda"),
                        mask=torch.empty((B, Hkv), dtype=torch.uint8, device="cuda")))
    torch.cuda.synchronize()

    def call(c):
        binding.sinkrouter_decode(c["q"], c["k"], c["v"], c["sl"], c["p"], c["out"], c["mask"])

    alone = []
    for c in ctx:                                 # one after the other
        call(c)
        torch.cuda.synchronize()
        alone.append((c["out"].clone(), c["mask"].clone()))
        c["out"].fill_(-1)
        c["mask"].fill_(9)
    torch.cuda.synchronize()
    for rep in range(5):                          # interleaved, no synchronisation in between
        for c in ctx:
            call(c)
    torch.cuda.synchronize()
    for c, (o, m) in zip(ctx, alone):
        assert torch.equal(c["out"], o) and torch.equal(c["mask"], m)
    assert not torch.equal(alone[0][0], alone[1][0])
