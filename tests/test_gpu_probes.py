"""The measurement helpers really move what they claim: the read probe touches every 16-byte word exactly
once (its XOR equals the buffer's), the copy probe copies (needs an MI355X)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2604_16883_amd import binding


@pytest.mark.parametrize("nbytes", [16, 4096, 16 * 1024 * 37 + 48, (1 << 26) + 16 * 5])
def test_read_probe_reads_every_word_once(nbytes):
    import torch
    rng = np.random.default_rng(nbytes)
    host = rng.integers(0, 2 ** 32, size=nbytes // 4, dtype=np.uint32)
    buf = torch.from_numpy(host.view(np.int32)).cuda()
    sink = torch.zeros((1024,), dtype=torch.int32, device="cuda")
    binding.sinkrouter_hbm_read_probe(buf, nbytes, sink)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    assert got == np.bitwise_xor.reduce(host)


def test_copy_probe_copies():
    import torch
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (1 << 20,), dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    binding.sinkrouter_hbm_copy_probe(dst, src, src.numel() * 4)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


def test_profiled_entry_gives_the_same_result_and_sane_times():
    """sinkrouter_decode_profiled launches the same kernels (with events attached): identical output
    bits; the separate probe is timed only when it is launched; the call span covers the kernels."""
    import oracle
    from paper_2604_16883_amd import synth
    import gpu_util as gu
    cases = [(synth.WORKLOADS["c0"].scaled(3000), dict(), True),                       # fused probe
             (synth.Workload("wide", 20, 32, 8, 300, 0.6, base_seed=91), dict(), False),   # separate probe, balanced
             (synth.WORKLOADS["c0"].scaled(3000), dict(num_splits=4), False)]          # separate probe, fixed chunks
    for w, kw, fused in cases:
        sb = synth.generate(w)
        plain = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, **kw)
        prof = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens, profiled=True, dev=plain["dev"], **kw)
        assert np.array_equal(plain["out_bits"], prof["out_bits"]) and np.array_equal(plain["mask"], prof["mask"])
        gu.compare(prof, oracle.decode(sb.q, sb.k, sb.v, sb.seq_lens, want_dense=True), w.group_size, "profiled " + w.name)
        probe, partial, merge, span = prof["stage_us"]
        assert (probe == 0.0) == fused, prof["stage_us"]
        assert 1.0 < partial < 1000.0 and 0.5 < merge < 100.0, prof["stage_us"]
        assert span >= partial + merge, prof["stage_us"]
        print(w.name, kw, "stage_us", [round(x, 2) for x in prof["stage_us"]], flush=True)
