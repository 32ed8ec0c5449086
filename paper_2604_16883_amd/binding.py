"""Thin ctypes binding of ``libsinkrouter.so``: argument marshalling only.

Functions carry the names of the C ABI (include/sinkrouter.h).  Tensor arguments
are torch tensors on the GPU (or anything with ``data_ptr()``), or raw integer
addresses; PyTorch is used for device memory and streams, every step of the path
runs in the library's kernels.  There is no fallback: if the library has not been
built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
# SINKROUTER_LIB selects another build of the same library (kernel tuning experiments)
LIB_PATH = os.environ.get("SINKROUTER_LIB") or os.path.join(HERE, "libsinkrouter.so")

SR_OK = 0
SR_ERR_NULL = -1
SR_ERR_SHAPE = -2
SR_ERR_UNSUPPORTED = -3
SR_ERR_WORKSPACE = -4
SR_ERR_ALIGN = -5
SR_ERR_HIP = -6
SR_ERR_STATIC_LIMIT = -7
STATIC_SCRATCH_BYTES = 32 << 20


class RouteParams(ctypes.Structure):
    """Mirror of ``sr_route_params``."""
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("batch", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("max_seq_len", ctypes.c_int32),
        ("kv_block", ctypes.c_int32),
        ("num_splits", ctypes.c_int32),
        ("routing_enabled", ctypes.c_int32),
        ("sm_scale", ctypes.c_float),
        ("tau_coef", ctypes.c_float * 4),
        ("len_norm", ctypes.c_float),
        ("k0_norm", ctypes.c_void_p),
        ("k0", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
    ]


class PagedLayout(ctypes.Structure):
    """Mirror of ``sr_paged_layout``."""
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("page_tokens", ctypes.c_int32),
        ("pages_per_seq", ctypes.c_int32),
        ("n_pages", ctypes.c_int32),
    ]


class Plan(ctypes.Structure):
    """Mirror of ``sr_plan``."""
    _fields_ = [
        ("schedule", ctypes.c_int32),
        ("chunk_tokens", ctypes.c_int32),
        ("num_splits", ctypes.c_int32),
        ("group_size", ctypes.c_int32),
        ("partial_grid", ctypes.c_int32),
        ("slots_per_head", ctypes.c_int32),
        ("workspace_bytes", ctypes.c_size_t),
    ]


class SinkRouterError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, sinkrouter_status_string(status), status))


_lib = None


def load() -> ctypes.CDLL:
    """Load the library built by ``paper_2604_16883_amd.build``; raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not found: build it first (python -m paper_2604_16883_amd.build or "
                "__graft_entry__.build()); there is no CPU fallback" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32p = ctypes.c_void_p, ctypes.c_void_p
        pp = ctypes.POINTER(RouteParams)
        lib.sinkrouter_plan.argtypes = [pp, ctypes.POINTER(Plan)]
        lib.sinkrouter_plan.restype = ctypes.c_int
        lib.sinkrouter_workspace_bytes.argtypes = [pp]
        lib.sinkrouter_workspace_bytes.restype = ctypes.c_size_t
        lib.sinkrouter_decode.argtypes = [vp, vp, vp, i32p, pp, vp, vp]
        lib.sinkrouter_decode.restype = ctypes.c_int
        lib.sinkrouter_decode_static.argtypes = [vp, vp, vp, i32p, pp, vp, vp]
        lib.sinkrouter_decode_static.restype = ctypes.c_int
        lib.sinkrouter_decode_profiled.argtypes = [vp, vp, vp, i32p, pp, vp, vp, ctypes.POINTER(ctypes.c_float)]
        lib.sinkrouter_decode_profiled.restype = ctypes.c_int
        lib.sinkrouter_decode_diag.argtypes = [vp, vp, vp, i32p, pp, vp, vp, vp, vp]
        lib.sinkrouter_decode_diag.restype = ctypes.c_int
        lib.sinkrouter_concentration.argtypes = [vp, vp, vp, i32p, pp, vp, vp, vp, vp, vp]
        lib.sinkrouter_concentration.restype = ctypes.c_int
        lib.sinkrouter_decode_paged.argtypes = [vp, vp, vp, vp, i32p, pp, ctypes.POINTER(PagedLayout), vp, vp]
        lib.sinkrouter_decode_paged.restype = ctypes.c_int
        lib.sinkrouter_extract_anchor.argtypes = [vp, pp, vp, vp]
        lib.sinkrouter_extract_anchor.restype = ctypes.c_int
        lib.sinkrouter_probe.argtypes = [vp, vp, i32p, pp, vp, vp]
        lib.sinkrouter_probe.restype = ctypes.c_int
        lib.sinkrouter_hbm_read_probe.argtypes = [vp, ctypes.c_size_t, vp, vp]
        lib.sinkrouter_hbm_read_probe.restype = ctypes.c_int
        lib.sinkrouter_hbm_copy_probe.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.sinkrouter_hbm_copy_probe.restype = ctypes.c_int
        lib.sinkrouter_timeline_bytes.argtypes = []
        lib.sinkrouter_timeline_bytes.restype = ctypes.c_size_t
        lib.sinkrouter_status_string.argtypes = [ctypes.c_int]
        lib.sinkrouter_status_string.restype = ctypes.c_char_p
        lib.sinkrouter_abi_version.argtypes = []
        lib.sinkrouter_abi_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def _addr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _current_stream() -> int:
    """torch's current stream on a GPU machine; the NULL (default) stream where there is no GPU,
    so that argument-error paths can be exercised without one."""
    import torch
    if not torch.cuda.is_available():
        return 0
    return int(torch.cuda.current_stream().cuda_stream)


def make_route_params(batch: int, n_q_heads: int, n_kv_heads: int, max_seq_len: int, *,
                      head_dim: int = 128, kv_block: int = 64, num_splits: int = 0,
                      routing_enabled: bool = True, sm_scale: float = 0.0,
                      tau_coef: Sequence[float] = (0.0, 0.0, 0.0, 0.55), len_norm: float = 0.0,
                      k0_norm=None, k0=None, workspace=None, workspace_bytes: Optional[int] = None,
                      stream: Optional[int] = None) -> RouteParams:
    """Fill an ``sr_route_params``.  ``workspace`` is a device tensor (kept alive by the caller)."""
    p = RouteParams()
    p.struct_size = ctypes.sizeof(RouteParams)
    p.batch, p.n_q_heads, p.n_kv_heads = int(batch), int(n_q_heads), int(n_kv_heads)
    p.head_dim, p.max_seq_len, p.kv_block = int(head_dim), int(max_seq_len), int(kv_block)
    p.num_splits = int(num_splits)
    p.routing_enabled = int(bool(routing_enabled))
    p.sm_scale = float(sm_scale)
    for i in range(4):
        p.tau_coef[i] = float(tau_coef[i])
    p.len_norm = float(len_norm)
    p.k0_norm = _addr(k0_norm)
    p.k0 = _addr(k0)
    p.workspace = _addr(workspace)
    if workspace_bytes is None and workspace is not None and not isinstance(workspace, int):
        workspace_bytes = workspace.numel() * workspace.element_size()
    p.workspace_bytes = int(workspace_bytes or 0)
    p.stream = stream
    return p


def sinkrouter_status_string(status: int) -> str:
    return load().sinkrouter_status_string(int(status)).decode()


def sinkrouter_timeline_bytes() -> int:
    return int(load().sinkrouter_timeline_bytes())


def sinkrouter_abi_version() -> int:
    return int(load().sinkrouter_abi_version())


def sinkrouter_plan(params: RouteParams) -> Plan:
    plan = Plan()
    rc = load().sinkrouter_plan(ctypes.byref(params), ctypes.byref(plan))
    if rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_plan")
    return plan


def sinkrouter_workspace_bytes(params: RouteParams) -> int:
    return int(load().sinkrouter_workspace_bytes(ctypes.byref(params)))


def _with_stream(params: RouteParams) -> RouteParams:
    if params.stream is None:
        q = RouteParams.from_buffer_copy(params)
        q.stream = _current_stream()
        return q
    return params


def sinkrouter_decode(q, k_cache, v_cache, seq_lens, route_params: RouteParams, out, skip_mask_out,
                      check: bool = True) -> int:
    """Enqueue one routed decode step; asynchronous.  With a NULL stream in ``route_params`` torch's
    current stream is used."""
    p = _with_stream(route_params)
    rc = load().sinkrouter_decode(_addr(q), _addr(k_cache), _addr(v_cache), _addr(seq_lens),
                                  ctypes.byref(p), _addr(out), _addr(skip_mask_out))
    if check and rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_decode")
    return rc


def sinkrouter_decode_static(q, k_cache, v_cache, seq_lens, route_params: RouteParams, out, skip_mask_out,
                             check: bool = True) -> int:
    """sinkrouter_decode on the library's own static scratch: no workspace, nothing allocated."""
    p = _with_stream(route_params)
    rc = load().sinkrouter_decode_static(_addr(q), _addr(k_cache), _addr(v_cache), _addr(seq_lens),
                                         ctypes.byref(p), _addr(out), _addr(skip_mask_out))
    if check and rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_decode_static")
    return rc


def sinkrouter_decode_profiled(q, k_cache, v_cache, seq_lens, route_params: RouteParams, out, skip_mask_out):
    """As sinkrouter_decode, synchronous; returns (probe_us, partial_us, combine_us, total_us)."""
    p = _with_stream(route_params)
    us = (ctypes.c_float * 4)()
    rc = load().sinkrouter_decode_profiled(_addr(q), _addr(k_cache), _addr(v_cache), _addr(seq_lens),
                                           ctypes.byref(p), _addr(out), _addr(skip_mask_out), us)
    if rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_decode_profiled")
    return tuple(float(x) for x in us)


def sinkrouter_decode_diag(q, k_cache, v_cache, seq_lens, route_params: RouteParams, out, skip_mask_out,
                           lse_out, alpha0_out, check: bool = True) -> int:
    """sinkrouter_decode plus per-head log-sum-exp and token-0 softmax mass (either may be None)."""
    p = _with_stream(route_params)
    rc = load().sinkrouter_decode_diag(_addr(q), _addr(k_cache), _addr(v_cache), _addr(seq_lens), ctypes.byref(p),
                                       _addr(out), _addr(skip_mask_out), _addr(lse_out), _addr(alpha0_out))
    if check and rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_decode_diag")
    return rc


def sinkrouter_concentration(q, k_cache, v_cache, seq_lens, route_params: RouteParams, out_rest, skip_mask_out,
                             alpha0_out, max_rest_out, mean_rest_out, check: bool = True) -> int:
    """Per-head weight of token 0, largest and mean weight of the other tokens, and the head update
    without token 0 (Section 3, Table 1); routing is ignored."""
    p = _with_stream(route_params)
    rc = load().sinkrouter_concentration(_addr(q), _addr(k_cache), _addr(v_cache), _addr(seq_lens), ctypes.byref(p),
                                         _addr(out_rest), _addr(skip_mask_out), _addr(alpha0_out),
                                         _addr(max_rest_out), _addr(mean_rest_out))
    if check and rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_concentration")
    return rc


def make_paged_layout(page_tokens: int, pages_per_seq: int, n_pages: int) -> PagedLayout:
    lay = PagedLayout()
    lay.struct_size = ctypes.sizeof(PagedLayout)
    lay.page_tokens, lay.pages_per_seq, lay.n_pages = int(page_tokens), int(pages_per_seq), int(n_pages)
    return lay


def sinkrouter_decode_paged(q, k_pages, v_pages, block_table, seq_lens, route_params: RouteParams,
                            layout: PagedLayout, out, skip_mask_out, check: bool = True) -> int:
    """One routed decode step over a paged KV cache; asynchronous."""
    p = _with_stream(route_params)
    rc = load().sinkrouter_decode_paged(_addr(q), _addr(k_pages), _addr(v_pages), _addr(block_table), _addr(seq_lens),
                                        ctypes.byref(p), ctypes.byref(layout), _addr(out), _addr(skip_mask_out))
    if check and rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_decode_paged")
    return rc


def sinkrouter_extract_anchor(k_cache, route_params: RouteParams, k0_out, k0_norm_out, check: bool = True) -> int:
    """Copy the token-0 keys and their norms out of the cache (prefill-side anchor caching)."""
    p = _with_stream(route_params)
    rc = load().sinkrouter_extract_anchor(_addr(k_cache), ctypes.byref(p), _addr(k0_out), _addr(k0_norm_out))
    if check and rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_extract_anchor")
    return rc


def sinkrouter_probe(q, k_cache, seq_lens, route_params: RouteParams, group_score_out, skip_mask_out,
                     check: bool = True) -> int:
    p = _with_stream(route_params)
    rc = load().sinkrouter_probe(_addr(q), _addr(k_cache), _addr(seq_lens), ctypes.byref(p),
                                 _addr(group_score_out), _addr(skip_mask_out))
    if check and rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_probe")
    return rc


def sinkrouter_hbm_read_probe(buf, nbytes: int, sink, stream: Optional[int] = None) -> int:
    rc = load().sinkrouter_hbm_read_probe(_addr(buf), int(nbytes), _addr(sink),
                                          _current_stream() if stream is None else stream)
    if rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_hbm_read_probe")
    return rc


def sinkrouter_hbm_copy_probe(dst, src, nbytes: int, stream: Optional[int] = None) -> int:
    rc = load().sinkrouter_hbm_copy_probe(_addr(dst), _addr(src), int(nbytes),
                                          _current_stream() if stream is None else stream)
    if rc != SR_OK:
        raise SinkRouterError(rc, "sinkrouter_hbm_copy_probe")
    return rc
