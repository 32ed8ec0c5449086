"""ctypes front end of the CPU oracle (``sr_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by
the benchmark's ``cpu_baseline`` leg.  It never imports the product package
and the product package never imports it.

Arrays are numpy; bf16 tensors travel as ``uint16`` bit patterns.  The oracle
returns fp64 results.  See the header of ``sr_oracle.c`` for what is computed
and which passage of the paper (Sections 3, 4.2, 4.3, Appendix A) each part
follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sr_oracle.c")
_LIB = os.path.join(_HERE, "libsr_oracle.so")


def build(force: bool = False) -> str:
    """Compile ``sr_oracle.c`` with gcc (fp64, OpenMP); returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
               "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
               _SRC, "-o", tmp, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


class _Cfg(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("max_seq_len", ctypes.c_int32),
        ("routing_enabled", ctypes.c_int32),
        ("want_dense", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("sm_scale", ctypes.c_double),
        ("tau_coef", ctypes.c_double * 4),
        ("len_norm", ctypes.c_double),
    ]


_lib = None


def _load(path: Optional[str] = None):
    """Load the oracle library (built on demand); ``path`` loads another build of it
    (the mutation tests compile deliberately broken copies of the source)."""
    global _lib
    if path is not None:
        lib = ctypes.CDLL(path)
        assert lib.sr_oracle_cfg_size() == ctypes.sizeof(_Cfg)
        return lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        assert lib.sr_oracle_cfg_size() == ctypes.sizeof(_Cfg)
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().sr_oracle_threads())


@dataclass
class OracleResult:
    out: np.ndarray                      # [B,Hq,D] fp64; zeros for Sink Groups
    mask: np.ndarray                     # [B,Hkv] uint8; 1 = Sink Group
    head_cos: np.ndarray                 # [B,Hq]  s_{g,i}
    group_score: np.ndarray              # [B,Hkv] S_g
    tau: np.ndarray                      # [B]
    dense_out: Optional[np.ndarray] = None   # [B,Hq,D] attention ignoring routing
    alpha0: Optional[np.ndarray] = None      # [B,Hq] softmax mass on token 0
    lse: Optional[np.ndarray] = None         # [B,Hq]
    extra: dict = field(default_factory=dict)


def _u16(a, shape):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 tensors are passed as uint16 bit patterns")
    if tuple(a.shape) != tuple(shape):
        raise ValueError("shape %r, expected %r" % (a.shape, shape))
    return a


def _cfg(B, Hq, Hkv, D, Lmax, routing_enabled, want_dense, sm_scale, tau_coef, len_norm):
    c = _Cfg()
    c.batch, c.n_q_heads, c.n_kv_heads, c.head_dim, c.max_seq_len = B, Hq, Hkv, D, Lmax
    c.routing_enabled = int(bool(routing_enabled))
    c.want_dense = int(bool(want_dense))
    c.sm_scale = float(sm_scale)
    for i in range(4):
        c.tau_coef[i] = float(tau_coef[i])
    c.len_norm = float(len_norm)
    return c


_keep = []


def _anchors(k0, B, Hkv, D):
    """Optional separately cached token-0 keys [B,Hkv,D] (uint16 bf16 bits) as a C pointer."""
    if k0 is None:
        return None
    a = _u16(k0, (B, Hkv, D))
    _keep[:] = [a]          # keep the contiguous copy alive during the call
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _ptr(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty)) if a is not None else None


def decode(q, k_cache, v_cache, seq_lens, *, tau_coef: Sequence[float] = (0.0, 0.0, 0.0, 0.55),
           len_norm: float = 0.0, sm_scale: float = 0.0, routing_enabled: bool = True,
           k0_norm=None, k0=None, want_dense: bool = False, diagnostics: bool = True,
           libpath: Optional[str] = None) -> OracleResult:
    """Routed decode attention in fp64 (single pass over each head's scores).

    q [B,Hq,D], k_cache/v_cache [B,Hkv,Lmax,D] as uint16 bf16 bits,
    seq_lens [B] int32 (valid rows, current token included).
    """
    lib = _load(libpath)
    q = np.ascontiguousarray(q)
    B, Hq, D = q.shape
    k_cache = np.ascontiguousarray(k_cache)
    _, Hkv, Lmax, _ = k_cache.shape
    q = _u16(q, (B, Hq, D))
    k_cache = _u16(k_cache, (B, Hkv, Lmax, D))
    v_cache = _u16(v_cache, (B, Hkv, Lmax, D))
    sl = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    assert sl.shape == (B,)
    c = _cfg(B, Hq, Hkv, D, Lmax, routing_enabled, want_dense, sm_scale, tau_coef, len_norm)
    out = np.empty((B, Hq, D), np.float64)
    mask = np.empty((B, Hkv), np.uint8)
    head_cos = np.empty((B, Hq), np.float64)
    group_score = np.empty((B, Hkv), np.float64)
    tau = np.empty((B,), np.float64)
    dense = np.empty((B, Hq, D), np.float64) if diagnostics else None
    alpha0 = np.empty((B, Hq), np.float64) if diagnostics else None
    lse = np.empty((B, Hq), np.float64) if diagnostics else None
    kn = None
    if k0_norm is not None:
        kn = np.ascontiguousarray(np.asarray(k0_norm, dtype=np.float64))
        assert kn.shape == (B, Hkv)
    dp = ctypes.c_double
    rc = lib.sr_oracle_decode(
        _ptr(q, ctypes.c_uint16), _ptr(k_cache, ctypes.c_uint16), _ptr(v_cache, ctypes.c_uint16),
        _ptr(sl, ctypes.c_int32), _ptr(kn, dp), _anchors(k0, B, Hkv, D), ctypes.byref(c),
        _ptr(out, dp), _ptr(mask, ctypes.c_uint8), _ptr(head_cos, dp), _ptr(group_score, dp),
        _ptr(tau, dp), _ptr(dense, dp), _ptr(alpha0, dp), _ptr(lse, dp))
    if rc != 0:
        raise RuntimeError("sr_oracle_decode failed: %d" % rc)
    return OracleResult(out, mask, head_cos, group_score, tau, dense, alpha0, lse)


def route(q, k_cache, seq_lens, *, tau_coef=(0.0, 0.0, 0.0, 0.55), len_norm: float = 0.0,
          routing_enabled: bool = True, k0_norm=None, k0=None, libpath: Optional[str] = None) -> OracleResult:
    """Routing decision only (cosine, group mean, threshold); reads row 0 of k_cache."""
    lib = _load(libpath)
    q = np.ascontiguousarray(q)
    B, Hq, D = q.shape
    k_cache = np.ascontiguousarray(k_cache)
    _, Hkv, Lmax, _ = k_cache.shape
    q = _u16(q, (B, Hq, D))
    k_cache = _u16(k_cache, (B, Hkv, Lmax, D))
    sl = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    c = _cfg(B, Hq, Hkv, D, Lmax, routing_enabled, False, 0.0, tau_coef, len_norm)
    mask = np.empty((B, Hkv), np.uint8)
    head_cos = np.empty((B, Hq), np.float64)
    group_score = np.empty((B, Hkv), np.float64)
    tau = np.empty((B,), np.float64)
    kn = None
    if k0_norm is not None:
        kn = np.ascontiguousarray(np.asarray(k0_norm, dtype=np.float64))
    dp = ctypes.c_double
    rc = lib.sr_oracle_route(
        _ptr(q, ctypes.c_uint16), _ptr(k_cache, ctypes.c_uint16), _ptr(sl, ctypes.c_int32),
        _ptr(kn, dp), _anchors(k0, B, Hkv, D), ctypes.byref(c), _ptr(head_cos, dp), _ptr(group_score, dp),
        _ptr(tau, dp), _ptr(mask, ctypes.c_uint8))
    if rc != 0:
        raise RuntimeError("sr_oracle_route failed: %d" % rc)
    return OracleResult(np.zeros((0,)), mask, head_cos, group_score, tau)


def decode_splitk(q, k_cache, v_cache, seq_lens, bounds, *, tau_coef=(0.0, 0.0, 0.0, 0.55),
                  len_norm: float = 0.0, sm_scale: float = 0.0, routing_enabled: bool = True,
                  k0_norm=None, k0=None, libpath: Optional[str] = None):
    """Routed decode attention reached through Split-K partials and the log-sum-exp merge.

    bounds: non-decreasing ints, bounds[0] == 0, bounds[-1] >= max(seq_lens).
    Returns (out [B,Hq,D] fp64, mask, part_m [B,Hq,S], part_l [B,Hq,S]).
    """
    lib = _load(libpath)
    q = np.ascontiguousarray(q)
    B, Hq, D = q.shape
    k_cache = np.ascontiguousarray(k_cache)
    _, Hkv, Lmax, _ = k_cache.shape
    q = _u16(q, (B, Hq, D))
    k_cache = _u16(k_cache, (B, Hkv, Lmax, D))
    v_cache = _u16(v_cache, (B, Hkv, Lmax, D))
    sl = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    bnd = np.ascontiguousarray(np.asarray(bounds, dtype=np.int32))
    S = bnd.shape[0] - 1
    c = _cfg(B, Hq, Hkv, D, Lmax, routing_enabled, False, sm_scale, tau_coef, len_norm)
    out = np.empty((B, Hq, D), np.float64)
    mask = np.empty((B, Hkv), np.uint8)
    pm = np.empty((B, Hq, S), np.float64)
    pl = np.empty((B, Hq, S), np.float64)
    kn = None
    if k0_norm is not None:
        kn = np.ascontiguousarray(np.asarray(k0_norm, dtype=np.float64))
    dp = ctypes.c_double
    rc = lib.sr_oracle_decode_splitk(
        _ptr(q, ctypes.c_uint16), _ptr(k_cache, ctypes.c_uint16), _ptr(v_cache, ctypes.c_uint16),
        _ptr(sl, ctypes.c_int32), _ptr(kn, dp), _anchors(k0, B, Hkv, D), ctypes.byref(c), _ptr(bnd, ctypes.c_int32),
        ctypes.c_int32(S), _ptr(out, dp), _ptr(mask, ctypes.c_uint8), _ptr(pm, dp), _ptr(pl, dp))
    if rc != 0:
        raise RuntimeError("sr_oracle_decode_splitk failed: %d" % rc)
    return out, mask, pm, pl


def concentration(q, k_cache, v_cache, seq_lens, *, sm_scale: float = 0.0, libpath: Optional[str] = None):
    """Per-head attention-concentration statistics (Section 3, Table 1): the softmax weight of
    token 0, the largest and the mean weight of the other tokens, and the head update with token 0
    left out.  Returns (alpha0, max_rest, mean_rest [B,Hq], out_rest [B,Hq,D]) in fp64."""
    lib = _load(libpath)
    q = np.ascontiguousarray(q)
    B, Hq, D = q.shape
    k_cache = np.ascontiguousarray(k_cache)
    _, Hkv, Lmax, _ = k_cache.shape
    q = _u16(q, (B, Hq, D))
    k_cache = _u16(k_cache, (B, Hkv, Lmax, D))
    v_cache = _u16(v_cache, (B, Hkv, Lmax, D))
    sl = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    assert sl.shape == (B,)
    c = _cfg(B, Hq, Hkv, D, Lmax, False, False, sm_scale, (0.0, 0.0, 0.0, 0.0), 0.0)
    a0 = np.empty((B, Hq), np.float64)
    mx = np.empty((B, Hq), np.float64)
    mean = np.empty((B, Hq), np.float64)
    rest = np.empty((B, Hq, D), np.float64)
    dp = ctypes.c_double
    rc = lib.sr_oracle_concentration(
        _ptr(q, ctypes.c_uint16), _ptr(k_cache, ctypes.c_uint16), _ptr(v_cache, ctypes.c_uint16),
        _ptr(sl, ctypes.c_int32), ctypes.byref(c), _ptr(a0, dp), _ptr(mx, dp), _ptr(mean, dp), _ptr(rest, dp))
    if rc != 0:
        raise RuntimeError("sr_oracle_concentration failed: %d" % rc)
    return a0, mx, mean, rest


def gather_pages(pages, block_table, seq_lens, max_seq_len: int, libpath: Optional[str] = None) -> np.ndarray:
    """Paged pool [n_pages,Hkv,page_tokens,D] + block_table [B,pages_per_seq] -> contiguous cache
    [B,Hkv,max_seq_len,D] (rows beyond seq_lens[b] are zero)."""
    lib = _load(libpath)
    pages = np.ascontiguousarray(pages)
    n_pages, Hkv, pt, D = pages.shape
    pages = _u16(pages, pages.shape)
    tab = np.ascontiguousarray(np.asarray(block_table, dtype=np.int32))
    B, pps = tab.shape
    sl = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    cache = np.empty((B, Hkv, int(max_seq_len), D), np.uint16)
    rc = lib.sr_oracle_gather_pages(_ptr(pages, ctypes.c_uint16), _ptr(tab, ctypes.c_int32), _ptr(sl, ctypes.c_int32),
                                    ctypes.c_int32(B), ctypes.c_int32(Hkv), ctypes.c_int32(D), ctypes.c_int32(int(max_seq_len)),
                                    ctypes.c_int32(pt), ctypes.c_int32(pps), ctypes.c_int32(n_pages),
                                    _ptr(cache, ctypes.c_uint16))
    if rc != 0:
        raise RuntimeError("sr_oracle_gather_pages failed: %d" % rc)
    return cache


def decode_paged(q, k_pages, v_pages, block_table, seq_lens, max_seq_len: int, **kw) -> OracleResult:
    """Routed decode over a paged cache: the decode step on the gathered contiguous cache."""
    lib = kw.get("libpath")
    k = gather_pages(k_pages, block_table, seq_lens, max_seq_len, libpath=lib)
    v = gather_pages(v_pages, block_table, seq_lens, max_seq_len, libpath=lib)
    return decode(q, k, v, seq_lens, **kw)
