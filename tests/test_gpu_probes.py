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
