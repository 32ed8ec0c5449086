"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, its plan/workspace arithmetic is sane, and every argument error is reported
before any HIP call.  (Compute calls are exercised by the -m gpu tests only.)"""
import ctypes
import os
import re

import pytest

from paper_2604_16883_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sinkrouter.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sinkrouter_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = declared_functions()
    assert len(names) >= 12 and "sinkrouter_decode_static" in names
    for n in names:
        assert hasattr(lib, n), "libsinkrouter.so does not export %s" % n
    assert B.sinkrouter_abi_version() == 2


def test_binding_mirrors_header_structs():
    text = open(HEADER).read()
    body = re.search(r"typedef struct sr_route_params \{(.*?)\} sr_route_params;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(\w+)(?:\[\d+\])?;", body)
    assert fields == [f[0] for f in B.RouteParams._fields_]
    body = re.search(r"typedef struct sr_plan \{(.*?)\} sr_plan;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(\w+);", body)
    assert fields == [f[0] for f in B.Plan._fields_]
    # the library checks struct_size itself
    p = B.make_route_params(1, 32, 8, 4096)
    assert B.sinkrouter_workspace_bytes(p) > 0
    p.struct_size += 8
    assert B.sinkrouter_workspace_bytes(p) == 0


def test_status_strings():
    seen = set()
    for code in (B.SR_OK, B.SR_ERR_NULL, B.SR_ERR_SHAPE, B.SR_ERR_UNSUPPORTED, B.SR_ERR_WORKSPACE, B.SR_ERR_ALIGN, B.SR_ERR_HIP,
                 B.SR_ERR_STATIC_LIMIT):
        s = B.sinkrouter_status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert B.sinkrouter_status_string(-99) == "unknown status"


WORKLOAD_SHAPES = {"c0": (1, 32, 8, 4096), "c1": (4, 32, 8, 32768), "c2": (1, 32, 4, 200000),
                   "c3": (1, 64, 8, 524288), "c4": (2, 40, 40, 65536)}


@pytest.mark.parametrize("name", sorted(WORKLOAD_SHAPES))
def test_plan_balanced(name):
    b, hq, hkv, L = WORKLOAD_SHAPES[name]
    pl = B.sinkrouter_plan(B.make_route_params(b, hq, hkv, L))
    assert pl.schedule == 1 and pl.partial_grid == 256 and pl.group_size == hq // hkv
    blocks = (L + 63) // 64
    assert pl.slots_per_head == min(blocks, 257)
    heads = b * hq
    need = heads * pl.slots_per_head * (128 + 2) * 4
    assert need <= pl.workspace_bytes <= need + 4096 + 8 * (b * hkv + 3) + 4 * b * hkv + 4 * b + 1280
    assert B.sinkrouter_workspace_bytes(B.make_route_params(b, hq, hkv, L)) == pl.workspace_bytes


@pytest.mark.parametrize("num_splits,L,chunk,splits", [(1, 4096, 4096, 1), (3, 4096, 1536, 3), (64, 4096, 256, 16),
                                                       (7, 200000, 28672, 7), (200, 524288, 2816, 187)])
def test_plan_fixed(num_splits, L, chunk, splits):
    pl = B.sinkrouter_plan(B.make_route_params(2, 32, 8, L, num_splits=num_splits))
    assert pl.schedule == 0
    assert pl.chunk_tokens == chunk and pl.chunk_tokens % 256 == 0
    assert pl.num_splits == splits == (L + chunk - 1) // chunk
    assert pl.partial_grid == splits * 2 * 8 and pl.slots_per_head == splits


def test_plan_falls_back_to_fixed_chunks_for_many_groups():
    pl = B.sinkrouter_plan(B.make_route_params(512, 32, 8, 2048))      # 4096 (sequence, group) pairs
    assert pl.schedule == 0 and pl.num_splits >= 1


FAKE = dict(q=0x10000, k=0x20000, v=0x30000, sl=0x40000, out=0x50000, mask=0x60000, ws=0x70000)


def call(p=None, **over):
    a = dict(FAKE)
    a.update(over)
    if p is None:
        p = B.make_route_params(1, 32, 8, 4096, workspace=a["ws"], workspace_bytes=1 << 30)
    return B.sinkrouter_decode(a["q"], a["k"], a["v"], a["sl"], p, a["out"], a["mask"], check=False)


def test_null_pointers_are_rejected():
    for key in ("q", "k", "v", "sl", "out", "mask"):
        assert call(**{key: None}) == B.SR_ERR_NULL, key
    lib = B.load()
    assert lib.sinkrouter_decode(1 << 16, 1 << 17, 1 << 18, 1 << 19, None, 1 << 20, 1 << 21) == B.SR_ERR_NULL
    assert lib.sinkrouter_plan(None, None) == B.SR_ERR_NULL
    p = B.make_route_params(1, 32, 8, 4096, workspace=FAKE["ws"], workspace_bytes=1 << 30)
    assert lib.sinkrouter_decode_profiled(1 << 16, 1 << 17, 1 << 18, 1 << 19, ctypes.byref(p), 1 << 20, 1 << 21, None) == B.SR_ERR_NULL
    assert B.sinkrouter_probe(None, FAKE["k"], FAKE["sl"], p, None, FAKE["mask"], check=False) == B.SR_ERR_NULL
    assert B.sinkrouter_probe(FAKE["q"], FAKE["k"], FAKE["sl"], p, None, None, check=False) == B.SR_ERR_NULL
    assert lib.sinkrouter_hbm_read_probe(None, 1024, 1 << 16, None) == B.SR_ERR_NULL
    # concentration statistics: all three statistic outputs are required, then the decode checks apply
    cargs = [FAKE["q"], FAKE["k"], FAKE["v"], FAKE["sl"], p, FAKE["out"], FAKE["mask"]]
    assert B.sinkrouter_concentration(*cargs, 1 << 22, None, 1 << 23, check=False) == B.SR_ERR_NULL
    assert B.sinkrouter_concentration(*cargs, None, 1 << 22, 1 << 23, check=False) == B.SR_ERR_NULL
    assert B.sinkrouter_concentration(FAKE["q"], None, FAKE["v"], FAKE["sl"], p, FAKE["out"], FAKE["mask"],
                                      1 << 22, 1 << 23, 1 << 24, check=False) == B.SR_ERR_NULL
    assert B.sinkrouter_concentration(*cargs, 1 << 22, (1 << 23) + 2, 1 << 24, check=False) == B.SR_ERR_ALIGN
    assert lib.sinkrouter_hbm_copy_probe(1 << 16, None, 1024, None) == B.SR_ERR_NULL


@pytest.mark.parametrize("kw,code", [
    (dict(batch=0), B.SR_ERR_SHAPE), (dict(n_q_heads=0), B.SR_ERR_SHAPE), (dict(n_kv_heads=0), B.SR_ERR_SHAPE),
    (dict(max_seq_len=0), B.SR_ERR_SHAPE), (dict(n_q_heads=33), B.SR_ERR_SHAPE), (dict(num_splits=-1), B.SR_ERR_SHAPE),
    (dict(max_seq_len=(1 << 24) + 1), B.SR_ERR_SHAPE), (dict(batch=70000, n_kv_heads=1, n_q_heads=1), B.SR_ERR_SHAPE),
    (dict(sm_scale=-1.0), B.SR_ERR_SHAPE), (dict(sm_scale=float("nan")), B.SR_ERR_SHAPE),
    (dict(head_dim=64), B.SR_ERR_UNSUPPORTED), (dict(kv_block=128), B.SR_ERR_UNSUPPORTED),
    (dict(n_q_heads=136, n_kv_heads=8), B.SR_ERR_UNSUPPORTED),
])
def test_bad_shapes(kw, code):
    base = dict(batch=1, n_q_heads=32, n_kv_heads=8, max_seq_len=4096, head_dim=128, kv_block=64, num_splits=0, sm_scale=0.0)
    base.update(kw)
    p = B.make_route_params(base["batch"], base["n_q_heads"], base["n_kv_heads"], base["max_seq_len"],
                            head_dim=base["head_dim"], kv_block=base["kv_block"], num_splits=base["num_splits"],
                            sm_scale=base["sm_scale"], workspace=FAKE["ws"], workspace_bytes=1 << 40)
    assert call(p) == code
    assert B.sinkrouter_workspace_bytes(p) == 0
    with pytest.raises(B.SinkRouterError) as e:
        B.sinkrouter_plan(p)
    assert e.value.status == code


def test_alignment_and_workspace_errors():
    for key in ("q", "k", "v", "out"):
        assert call(**{key: FAKE[key] + 8}) == B.SR_ERR_ALIGN, key
    assert call(sl=FAKE["sl"] + 2) == B.SR_ERR_ALIGN
    need = B.sinkrouter_workspace_bytes(B.make_route_params(1, 32, 8, 4096))
    assert call(B.make_route_params(1, 32, 8, 4096)) == B.SR_ERR_WORKSPACE                       # no workspace
    assert call(B.make_route_params(1, 32, 8, 4096, workspace=FAKE["ws"], workspace_bytes=need - 1)) == B.SR_ERR_WORKSPACE
    assert call(B.make_route_params(1, 32, 8, 4096, workspace=FAKE["ws"] + 128, workspace_bytes=need)) == B.SR_ERR_WORKSPACE
    lib = B.load()
    assert lib.sinkrouter_hbm_read_probe(1 << 16, 1000, 1 << 17, None) == B.SR_ERR_SHAPE
    assert lib.sinkrouter_hbm_read_probe((1 << 16) + 4, 1024, 1 << 17, None) == B.SR_ERR_ALIGN


def test_plan_rejects_a_fixed_grid_beyond_32_bits():
    # 65536 chunks of 256 tokens x 65535 groups: the workgroup count does not fit a 32-bit grid
    p = B.make_route_params(65535, 1, 1, 1 << 24, num_splits=65536)
    with pytest.raises(B.SinkRouterError) as e:
        B.sinkrouter_plan(p)
    assert e.value.status == B.SR_ERR_SHAPE
    assert B.sinkrouter_workspace_bytes(p) == 0
    pl = B.sinkrouter_plan(B.make_route_params(32767, 1, 1, 1 << 24, num_splits=65536))
    assert pl.partial_grid == 65536 * 32767 and pl.num_splits == 65536


def test_static_entry_point_checks_arguments_and_its_size_limit_on_the_host():
    """sinkrouter_decode_static takes no workspace; every check, the size limit included, precedes any HIP call."""
    args = (FAKE["q"], FAKE["k"], FAKE["v"], FAKE["sl"])
    ok = B.make_route_params(1, 32, 8, 4096)                         # no workspace given: fine here
    assert B.sinkrouter_plan(ok).workspace_bytes <= B.STATIC_SCRATCH_BYTES
    assert B.sinkrouter_decode_static(None, *args[1:], ok, FAKE["out"], FAKE["mask"], check=False) == B.SR_ERR_NULL
    assert B.sinkrouter_decode_static(FAKE["q"] + 8, *args[1:], ok, FAKE["out"], FAKE["mask"], check=False) == B.SR_ERR_ALIGN
    bad = B.make_route_params(1, 32, 8, 4096, head_dim=64)
    assert B.sinkrouter_decode_static(*args, bad, FAKE["out"], FAKE["mask"], check=False) == B.SR_ERR_UNSUPPORTED
    for name, (b, hq, hkv, L) in WORKLOAD_SHAPES.items():            # the five benchmark shapes fit
        assert B.sinkrouter_plan(B.make_route_params(b, hq, hkv, L)).workspace_bytes <= B.STATIC_SCRATCH_BYTES, name
    big = B.make_route_params(16, 32, 8, 32768)                      # 512 heads x 257 records: 68 MB
    assert B.sinkrouter_plan(big).workspace_bytes > B.STATIC_SCRATCH_BYTES
    assert B.sinkrouter_decode_static(*args, big, FAKE["out"], FAKE["mask"], check=False) == B.SR_ERR_STATIC_LIMIT
    assert "static scratch" in B.sinkrouter_status_string(B.SR_ERR_STATIC_LIMIT)
    text = open(HEADER).read()
    assert int(re.search(r"SINKROUTER_STATIC_SCRATCH_BYTES \(\(size_t\)(\d+) << 20\)", text).group(1)) << 20 == B.STATIC_SCRATCH_BYTES


def test_paged_argument_errors():
    p = B.make_route_params(1, 32, 8, 4096, workspace=0x70000, workspace_bytes=1 << 30)
    args = (0x10000, 0x20000, 0x30000, 0x80000, 0x40000)
    for lay, code in ((B.make_paged_layout(48, 100, 10), B.SR_ERR_UNSUPPORTED),
                      (B.make_paged_layout(32, 200, 10), B.SR_ERR_UNSUPPORTED),
                      (B.make_paged_layout(64, 10, 10), B.SR_ERR_SHAPE),
                      (B.make_paged_layout(64, 64, 0), B.SR_ERR_SHAPE)):
        assert B.sinkrouter_decode_paged(*args, p, lay, 0x50000, 0x60000, check=False) == code
    lay = B.make_paged_layout(64, 64, 10)
    assert B.sinkrouter_decode_paged(0x10000, 0x20000, 0x30000, None, 0x40000, p, lay, 0x50000, 0x60000, check=False) == B.SR_ERR_NULL
    lay.struct_size += 4
    assert B.sinkrouter_decode_paged(*args, p, lay, 0x50000, 0x60000, check=False) == B.SR_ERR_UNSUPPORTED


def test_compute_call_without_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    # valid arguments, no device: the HIP launch fails and the library says so; nothing falls back to the CPU
    assert call() == B.SR_ERR_HIP
    # the allocation-free entry point needs the device address of its scratch array: no device, no address
    assert B.sinkrouter_decode_static(FAKE["q"], FAKE["k"], FAKE["v"], FAKE["sl"], B.make_route_params(1, 32, 8, 4096),
                                      FAKE["out"], FAKE["mask"], check=False) == B.SR_ERR_HIP
    assert B.sinkrouter_timeline_bytes() == 0           # the product build carries no stamps
    with pytest.raises(B.SinkRouterError):
        B.sinkrouter_decode(FAKE["q"], FAKE["k"], FAKE["v"], FAKE["sl"],
                            B.make_route_params(1, 32, 8, 4096, workspace=FAKE["ws"], workspace_bytes=1 << 30),
                            FAKE["out"], FAKE["mask"])


def test_missing_library_raises(tmp_path, monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        B.load()


def test_header_is_plain_c(tmp_path):
    """The boundary header must compile as strict C99 and as C++ with no other include."""
    import subprocess
    src = tmp_path / "use.c"
    src.write_text('#include "sinkrouter.h"\n'
                   'int f(void) { sr_route_params p; sr_plan pl; sr_paged_layout lay; p.struct_size = sizeof p; lay.struct_size = sizeof lay;\n'
                   '  (void)lay; return sinkrouter_plan(&p, &pl) + (int)sizeof(sr_status) + SINKROUTER_ABI_VERSION; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    cpp = tmp_path / "use.cpp"
    cpp.write_text(src.read_text())
    subprocess.run(["g++", "-std=c++11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(cpp)], check=True)


def test_struct_sizes_match_the_c_compiler(tmp_path):
    """ctypes mirrors and the C compiler agree on sizes and field offsets."""
    import subprocess
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "sinkrouter.h"\n'
                   'int main(void) { printf("%zu %zu %zu %zu %zu %zu %zu\\n", sizeof(sr_route_params), offsetof(sr_route_params, tau_coef),\n'
                   '  offsetof(sr_route_params, k0_norm), offsetof(sr_route_params, workspace), offsetof(sr_route_params, stream),\n'
                   '  sizeof(sr_plan), sizeof(sr_paged_layout)); return 0; }\n')
    exe = tmp_path / "sizes"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    P = B.RouteParams
    assert got == [ctypes.sizeof(P), P.tau_coef.offset, P.k0_norm.offset, P.workspace.offset, P.stream.offset,
                   ctypes.sizeof(B.Plan), ctypes.sizeof(B.PagedLayout)]


@pytest.mark.parametrize("timeline", [False, True], ids=["product", "measurement"])
def test_both_library_variants_compile_without_register_spills(tmp_path, timeline):
    """The build script refuses a library whose kernels spill registers to scratch memory; the measurement variant
    (wall-clock stamps in the kernels) has its own register budget and must pass as well as the product one."""
    import shutil
    from paper_2604_16883_amd import build
    if not (os.path.exists(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")) or shutil.which("hipcc")):
        pytest.skip("no hipcc here")
    out = build.build_library(timeline=timeline, out=str(tmp_path / "lib.so"))
    lib = ctypes.CDLL(out)
    lib.sinkrouter_timeline_bytes.restype = ctypes.c_size_t
    assert (lib.sinkrouter_timeline_bytes() > 0) == timeline
