"""A stack of layers with routing switched off in the first two (Appendix B of the paper), eager and as one
HIP graph, against the oracle layer by layer (needs an MI355X)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2604_16883_amd import synth
from paper_2604_16883_amd.layers import LayerStack

import gpu_util as gu


def test_layer_stack_first_two_layers_dense():
    import torch
    n_layers = 5
    w = synth.WORKLOADS["c1"].scaled(1200, batch=2)
    batches = [synth.generate(w, seed=300 + l, seq_lens=[1200, 801]) for l in range(n_layers)]
    ks = [gu.to_dev(sb.k) for sb in batches]
    vs = [gu.to_dev(sb.v) for sb in batches]
    qs = [gu.to_dev(sb.q) for sb in batches]
    sl = gu.to_dev(batches[0].seq_lens)
    stack = LayerStack(ks, vs, sl, w.n_q_heads)
    stack.step(qs)
    torch.cuda.synchronize()
    eager = [o.clone() for o in stack.out]
    for l, sb in enumerate(batches):
        routed = l >= 2
        ref = oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, routing_enabled=routed, want_dense=True)
        bits = stack.out[l].cpu().numpy().view(np.uint16)
        res = dict(out=synth.bf16_bits_to_f32(bits), out_bits=bits, mask=stack.mask[l].cpu().numpy())
        res["probe_mask"], res["score"] = res["mask"], ref.group_score.astype(np.float32)
        rep = gu.compare(res, ref, w.group_size, "layer %d" % l)
        assert (rep["skip_ratio"] > 0) == routed, "layers 0 and 1 must not be routed"
        print("layer", l, rep, flush=True)
    # the whole stack as one graph
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        stack.step(qs)
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        stack.step(qs)
    for rep in range(3):
        for o in stack.out:
            o.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for l in range(n_layers):
            assert torch.equal(stack.out[l], eager[l])
