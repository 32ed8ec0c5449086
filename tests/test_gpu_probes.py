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


CHILD = r"""
import os, sys, json
import numpy as np, torch
sys.path.insert(0, sys.argv[1]); sys.path.insert(0, os.path.join(sys.argv[1], "tests"))
from paper_2604_16883_amd import binding, synth
import gpu_util as gu
w = synth.WORKLOADS["c1"].scaled(3000)
sb = synth.generate(w, seq_lens=[3000, 2933, 64, 1])
nb = binding.sinkrouter_timeline_bytes()
res = gu.run_hip(sb.q, sb.k, sb.v, sb.seq_lens)
# stamps of one more call on a zeroed workspace
B, Hq, Hkv, Lmax = w.batch, w.n_q_heads, w.n_kv_heads, sb.max_seq_len
p = binding.make_route_params(B, Hq, Hkv, Lmax)
plan = binding.sinkrouter_plan(p)
ws = torch.zeros((plan.workspace_bytes,), dtype=torch.uint8, device="cuda")
p.workspace, p.workspace_bytes = ws.data_ptr(), plan.workspace_bytes
out = torch.empty((B, Hq, 128), dtype=torch.int16, device="cuda"); mask = torch.empty((B, Hkv), dtype=torch.uint8, device="cuda")
d = res["dev"]
binding.sinkrouter_decode(d["q"], d["k"], d["v"], d["sl"], p, out, mask)
torch.cuda.synchronize()
t = ws[plan.workspace_bytes - nb:].cpu().numpy().view(np.int64) if nb else np.zeros((0,), np.int64)
np.savez(sys.argv[2], out_bits=res["out_bits"], mask=res["mask"], stamps=t, nb=nb, ws_bytes=plan.workspace_bytes,
         out2=out.cpu().numpy().view(np.uint16))
"""


def test_measurement_build_computes_the_same_bits_and_leaves_ordered_stamps(tmp_path):
    """The library built with -DSR_TIMELINE=1 (bench.py --timeline) differs from the product build only in the
    wall-clock stamps it leaves behind the workspace: same output bits, same mask; the stamps of every workgroup are
    in program order.  Run in a child process, since a process loads one build of the library."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    tl = os.path.join(root, "paper_2604_16883_amd", "libsinkrouter_timeline.so")
    if not os.path.exists(tl):
        pytest.skip("measurement build missing (python -m paper_2604_16883_amd.build --timeline)")
    got = {}
    for name, lib in (("product", ""), ("timeline", tl)):
        env = dict(os.environ)
        env.pop("SINKROUTER_LIB", None)
        if lib:
            env["SINKROUTER_LIB"] = lib
        path = str(tmp_path / (name + ".npz"))
        r = subprocess.run([sys.executable, "-c", CHILD, root, path], env=env, capture_output=True, text=True, timeout=300)
        assert r.returncode == 0, r.stderr[-3000:]
        got[name] = np.load(path)
    a, b = got["product"], got["timeline"]
    assert int(a["nb"]) == 0 and int(b["nb"]) == (256 * 8 + 1024 * 4) * 8
    assert int(b["ws_bytes"]) == int(a["ws_bytes"]) + int(b["nb"])
    assert np.array_equal(a["out_bits"], b["out_bits"]) and np.array_equal(a["mask"], b["mask"])
    assert np.array_equal(a["out2"], b["out2"]) and np.array_equal(a["out2"], a["out_bits"])
    tp = b["stamps"][:256 * 8].reshape(256, 8)
    tm = b["stamps"][256 * 8:].reshape(1024, 4)[:4 * 32]
    busy = tp[:, 5] > 0
    assert busy.any() and np.all(tp[:, 0] > 0)
    assert np.all(np.diff(tp[busy][:, [0, 1, 2, 3, 4, 5, 6, 7]], axis=1) >= 0)        # entry .. exit, in order
    assert np.all(np.diff(tp[~busy][:, [0, 1, 2, 3]], axis=1) >= 0)                    # idle workgroups stop after the schedule
    merged = tm[:, 1] > 0
    assert merged.any() and np.all(np.diff(tm[merged], axis=1) >= 0)
    assert np.all(tm[~merged][:, 3] >= tm[~merged][:, 0])
    assert tm[:, 0].min() >= tp[:, 7].max()                                            # the merge starts after the last partial exit
    assert (tm[:, 3].max() - tp[:, 0].min()) / 100.0 < 200.0                           # the whole step, in microseconds
