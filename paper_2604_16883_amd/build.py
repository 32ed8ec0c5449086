"""Builds ``libsinkrouter.so`` (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "sinkrouter.hip")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(HERE, "libsinkrouter.so")
# measurement variant (wall-clock stamps per workgroup, -DSR_TIMELINE=1); only bench.py --timeline loads it
TIMELINE_LIB = os.path.join(HERE, "libsinkrouter_timeline.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    # one remark block per kernel with its register, LDS and scratch use (checked below)
    "-Rpass-analysis=kernel-resource-usage",
]


def build_library(verbose: bool = False, extra=(), timeline: bool = False, out: str = "") -> str:
    """Compile the library (or, with ``timeline``, its measurement variant) unconditionally; returns its path
    (``out`` if given, else the in-tree location).  Raises if hipcc fails or any kernel spills registers."""
    LIB = out or (TIMELINE_LIB if timeline else globals()["LIB"])
    extra = list(extra) + (["-DSR_TIMELINE=1"] if timeline else [])
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + ["-I", INCLUDE, SRC, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass prints one harmless line per target feature it does not know
    log = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + log)
    usage = kernel_resource_usage(log)
    import re
    keep, skip = [], 0
    for l in log.splitlines():          # drop the remarks and the two source-echo lines after each
        if "[-Rpass-analysis=kernel-resource-usage]" in l:
            skip = 2
        elif skip and re.match(r"^\s+(\d+ )?\|", l):
            skip -= 1
        else:
            skip = 0
            keep.append(l)
    log = "\n".join(keep)
    if verbose and log.strip():
        print(log)
    if verbose:
        for name, u in sorted(usage.items()):
            print("  %-60s VGPRs %3s  LDS %6s B  scratch %s B/lane" % (name[:60], u.get("VGPRs"), u.get("LDS Size [bytes/block]"),
                                                                      u.get("ScratchSize [bytes/lane]")))
    spilled = [n for n, u in usage.items() if int(u.get("ScratchSize [bytes/lane]", 0)) > 0]
    if spilled:
        os.remove(tmp)
        raise RuntimeError("kernels spill registers to scratch memory: %s" % ", ".join(spilled))
    os.replace(tmp, LIB)
    return LIB


def ensure_built() -> str:
    """For the tests, the smoke check and the benchmark: the library as it stands if it has been built, else one
    build now.  (The binding itself never builds and never falls back: without the library it raises.)"""
    if not os.path.exists(LIB):
        build_library()
    return LIB


def kernel_resource_usage(log: str) -> dict:
    """Parse clang's kernel-resource-usage remarks: {kernel name: {field: value}}."""
    import re
    usage, cur = {}, None
    for line in log.splitlines():
        m = re.search(r"remark: Function Name: (\S+) \[-Rpass-analysis", line)
        if m:
            cur = usage.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z][^:]*): (\S+) \[-Rpass-analysis", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = m.group(2)
    return usage


if __name__ == "__main__":
    args = sys.argv[1:]
    tl = "--timeline" in args
    print(build_library(verbose=True, extra=[a for a in args if a != "--timeline"], timeline=tl))
