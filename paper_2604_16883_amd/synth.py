"""Seeded synthetic decode-attention inputs shaped like the paper's backbones.

This module serves the tests, the smoke check and the benchmark, for both the
CPU oracle and the HIP path.  It holds only input construction: random draws,
bf16 rounding and the planting of sink / retrieval structure.  None of the
method's arithmetic (routing signal, threshold, softmax, Split-K) lives here,
and it imports neither the oracle nor the HIP binding.

The caches stand in for KV caches that the paper obtains by running long
prompts through Llama-3.1-8B/70B, Yi-9B-200K and LLaVA-1.5 (Section 5.1); only
their shapes and the sink structure the paper reports (a near-zero value at
token 0, Section 3 / Fig. 1, and queries aligned in direction with the token-0
key, Section 3 / Eq. 6) are reproduced.

Recipe, per (sequence b, KV group g), everything drawn from numpy PCG64
streams keyed by (seed, tensor, b, g) so the result does not depend on thread
count or generation order:
  * Q, K, V ~ N(0, 1) in fp32, rounded once to bf16 (round to nearest even).
  * each query head is "sink-dominated" with probability ``sink_frac``
    (seeded Bernoulli per head); such a head gets ``q += sink_gain * u_g`` for
    a unit direction u_g of the group.
  * K[b,g,0] = anchor_norm * normalise(mean of the group's sink-head queries)
    (u_g if the group has none); V[b,g,0] = anchor_value_norm * unit vector.
  * every other head gets ``planted_per_head`` seeded positions in [1, L)
    whose key is ``planted_gain * q_h / ||q_h||`` so they carry its mass.
  * ``secondary_sinks`` extra early positions (< 64) whose key is
    ``secondary_gain`` times the anchor direction and whose value norm is
    anchor_value_norm (routing must ignore them: it reads token 0 only).
  * ``image_segments`` non-overlapping runs of ``image_len`` tokens whose K/V
    are N(0, image_sigma^2) (multimodal layer).
  * rows at or beyond seq_lens[b] are filled with NaN bit patterns ("poison")
    so any read past the valid length shows up in the output.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

BF16_NAN = np.uint16(0x7FC0)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even. NaN stays NaN."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r[nan] = BF16_NAN
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32, exact."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    seq_len: int
    sink_frac: float
    head_dim: int = 128
    kv_block: int = 64
    sink_gain: float = 32.0
    anchor_norm: float = 8.0
    anchor_value_norm: float = 0.01
    planted_per_head: int = 16
    planted_gain: float = 16.0
    secondary_sinks: int = 0
    secondary_gain: float = 6.0
    image_segments: int = 0
    image_len: int = 576
    image_sigma: float = 1.5
    n_taus: int = 1
    base_seed: int = 0
    description: str = ""

    @property
    def group_size(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def scaled(self, seq_len: int, batch: Optional[int] = None, name: Optional[str] = None) -> "Workload":
        """Same recipe at another context length (reduced-size parity cases)."""
        return dataclasses.replace(self, seq_len=int(seq_len),
                                   batch=self.batch if batch is None else int(batch),
                                   name=name or "%s@L%d" % (self.name, seq_len))

    def dense_kv_bytes(self) -> int:
        return self.batch * self.n_kv_heads * self.seq_len * self.head_dim * 2 * 2


# The five workloads: single layer, one decode step, bf16, KV block 64.
WORKLOADS: Dict[str, Workload] = {
    "c0": Workload("c0", 1, 32, 8, 4096, 0.7, base_seed=0,
                   description="Llama-3.1-8B-shaped layer, B1, 32/8 heads, L 4096"),
    "c1": Workload("c1", 4, 32, 8, 32768, 0.7, n_taus=3, base_seed=1000,
                   description="Llama-3.1-8B-shaped layer, B4, 32/8 heads, L 32768 each (128K tokens)"),
    "c2": Workload("c2", 1, 32, 4, 200000, 0.6, secondary_sinks=4, base_seed=2000,
                   description="Yi-9B-200K-shaped layer, B1, 32/4 heads, L 200000"),
    "c3": Workload("c3", 1, 64, 8, 524288, 0.7, base_seed=3000,
                   description="Llama-3.1-70B-shaped layer, B1, 64/8 heads, L 524288 (512K)"),
    "c4": Workload("c4", 2, 40, 40, 65536, 0.5, image_segments=8, base_seed=4000,
                   description="LLaVA-1.5-13B-shaped layer, B2, 40 MHA heads, L 65536, 8 image segments"),
}


@dataclass
class SynthBatch:
    workload: Workload
    seed: int
    q: np.ndarray            # [B,Hq,D] uint16 (bf16 bits)
    k: np.ndarray            # [B,Hkv,Lmax,D] uint16
    v: np.ndarray            # [B,Hkv,Lmax,D] uint16
    seq_lens: np.ndarray     # [B] int32
    sink_head: np.ndarray    # [B,Hq] bool: planted as sink-dominated
    taus: Tuple[float, ...]  # thresholds to run (first is the operating point 0.55)
    planted_pos: Dict[Tuple[int, int], np.ndarray]   # (b,h) -> positions, non-sink heads
    secondary_pos: Dict[Tuple[int, int], np.ndarray]  # (b,g) -> positions
    image_starts: Dict[int, np.ndarray]              # b -> segment starts

    @property
    def max_seq_len(self) -> int:
        return int(self.k.shape[2])


def _rng(seed: int, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed)] + [int(x) for x in key])))


def _unit(rng: np.random.Generator, D: int) -> np.ndarray:
    x = rng.standard_normal(D).astype(np.float32)
    return x / np.linalg.norm(x)


_SLAB_ROWS = 1 << 15


def _fill_normal_bf16(dst: np.ndarray, rng: np.random.Generator, sigma_rows: Optional[np.ndarray]) -> None:
    """dst[L,D] uint16 <- bf16(N(0,1) * sigma_rows[:,None]), generated in row slabs."""
    L, D = dst.shape
    for r0 in range(0, L, _SLAB_ROWS):
        r1 = min(L, r0 + _SLAB_ROWS)
        x = rng.standard_normal((r1 - r0, D), dtype=np.float32)
        if sigma_rows is not None:
            x *= sigma_rows[r0:r1, None]
        dst[r0:r1] = f32_to_bf16_bits(x)


def generate(w: Workload, seed: Optional[int] = None, seq_lens: Optional[Sequence[int]] = None,
             max_seq_len: Optional[int] = None, threads: int = 8) -> SynthBatch:
    """Build one decode step's inputs for workload ``w``.

    seq_lens defaults to ``w.seq_len`` for every sequence; ``max_seq_len`` (the
    cache's token stride) defaults to max(seq_lens).
    """
    seed = w.base_seed if seed is None else int(seed)
    B, Hq, Hkv, D = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    G = Hq // Hkv
    assert Hq % Hkv == 0
    sl = np.full((B,), w.seq_len, np.int32) if seq_lens is None else np.asarray(seq_lens, np.int32)
    assert sl.shape == (B,)
    Lmax = int(max(1, sl.max())) if max_seq_len is None else int(max_seq_len)
    assert Lmax >= int(sl.max())

    # --- queries and the sink-head choice -------------------------------------------------
    rq = _rng(seed, 1)
    q32 = rq.standard_normal((B, Hq, D)).astype(np.float32)
    sink_head = _rng(seed, 2).random((B, Hq)) < w.sink_frac
    u = np.stack([[_unit(_rng(seed, 3, b, g), D) for g in range(Hkv)] for b in range(B)])  # [B,Hkv,D]
    for b in range(B):
        for h in range(Hq):
            if sink_head[b, h]:
                q32[b, h] += np.float32(w.sink_gain) * u[b, h // G]
    q_bits = f32_to_bf16_bits(q32)
    qf = bf16_bits_to_f32(q_bits)            # the values both sides will actually see

    # --- image segments (per sequence) ----------------------------------------------------
    image_starts: Dict[int, np.ndarray] = {}
    sigma_rows: Dict[int, Optional[np.ndarray]] = {}
    for b in range(B):
        L = int(sl[b])
        sigma_rows[b] = None
        if w.image_segments > 0 and L > w.image_segments * w.image_len + 1:
            ri = _rng(seed, 4, b)
            # non-overlapping starts: draw gaps over the free text tokens
            free = L - 1 - w.image_segments * w.image_len
            cuts = np.sort(ri.integers(0, free + 1, size=w.image_segments))
            starts = 1 + cuts + np.arange(w.image_segments) * w.image_len
            image_starts[b] = starts.astype(np.int64)
            s = np.ones((Lmax,), np.float32)
            for st in starts:
                s[st:st + w.image_len] = np.float32(w.image_sigma)
            sigma_rows[b] = s

    # --- bulk K/V ------------------------------------------------------------------------
    k = np.empty((B, Hkv, Lmax, D), np.uint16)
    v = np.empty((B, Hkv, Lmax, D), np.uint16)

    def _bulk(job):
        which, b, g = job
        dst = (k if which == 0 else v)[b, g]
        L = int(sl[b])
        _fill_normal_bf16(dst[:L], _rng(seed, 10 + which, b, g), None if sigma_rows[b] is None else sigma_rows[b][:L])
        if L < Lmax:
            dst[L:] = BF16_NAN

    jobs = [(which, b, g) for which in (0, 1) for b in range(B) for g in range(Hkv)]
    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(_bulk, jobs))
    else:
        for j in jobs:
            _bulk(j)

    # --- planted structure ---------------------------------------------------------------
    planted_pos: Dict[Tuple[int, int], np.ndarray] = {}
    secondary_pos: Dict[Tuple[int, int], np.ndarray] = {}
    for b in range(B):
        L = int(sl[b])
        if L < 1:
            continue
        for g in range(Hkv):
            rp = _rng(seed, 5, b, g)
            heads = list(range(g * G, (g + 1) * G))
            sinks = [h for h in heads if sink_head[b, h]]
            if sinks:
                a = qf[b, sinks].mean(axis=0)
                a = a / np.linalg.norm(a)
            else:
                a = u[b, g]
            k[b, g, 0] = f32_to_bf16_bits(np.float32(w.anchor_norm) * a)
            v[b, g, 0] = f32_to_bf16_bits(np.float32(w.anchor_value_norm) * _unit(rp, D))
            taken = np.zeros((L,), bool)
            taken[0] = True
            if w.secondary_sinks > 0 and L > 1:
                hi = min(64, L)
                n = min(w.secondary_sinks, hi - 1)
                pos = 1 + rp.choice(hi - 1, size=n, replace=False)
                secondary_pos[(b, g)] = np.sort(pos)
                for p in pos:
                    k[b, g, p] = f32_to_bf16_bits(np.float32(w.secondary_gain) * a)
                    v[b, g, p] = f32_to_bf16_bits(np.float32(w.anchor_value_norm) * _unit(rp, D))
                    taken[p] = True
            for h in heads:
                if sink_head[b, h]:
                    continue
                freepos = np.flatnonzero(~taken)
                n = min(w.planted_per_head, freepos.size)
                if n == 0:
                    planted_pos[(b, h)] = np.zeros((0,), np.int64)
                    continue
                pos = rp.choice(freepos, size=n, replace=False)
                planted_pos[(b, h)] = np.sort(pos)
                key = np.float32(w.planted_gain) * qf[b, h] / np.linalg.norm(qf[b, h])
                kb = f32_to_bf16_bits(key)
                for p in pos:
                    k[b, g, p] = kb
                    taken[p] = True

    # --- thresholds ----------------------------------------------------------------------
    taus = [0.55]
    if w.n_taus > 1:
        rt = _rng(seed, 6)
        taus += [float(np.float32(t)) for t in rt.uniform(0.35, 0.75, size=w.n_taus)]
    return SynthBatch(w, seed, q_bits, k, v, sl, sink_head, tuple(taus), planted_pos, secondary_pos, image_starts)


def random_small(seed: int, B: int, Hq: int, Hkv: int, D: int, Lmax: int,
                 seq_lens: Optional[Sequence[int]] = None, scale: float = 1.0):
    """Plain N(0, scale^2) bf16 tensors of arbitrary small shape (oracle pins, edge cases).

    Returns (q, k, v, seq_lens) with rows beyond seq_lens poisoned with NaN.
    """
    r = _rng(seed, 99)
    q = f32_to_bf16_bits(r.standard_normal((B, Hq, D)).astype(np.float32) * np.float32(scale))
    k = f32_to_bf16_bits(r.standard_normal((B, Hkv, Lmax, D)).astype(np.float32) * np.float32(scale))
    v = f32_to_bf16_bits(r.standard_normal((B, Hkv, Lmax, D)).astype(np.float32) * np.float32(scale))
    sl = np.full((B,), Lmax, np.int32) if seq_lens is None else np.asarray(seq_lens, np.int32)
    for b in range(B):
        k[b, :, int(sl[b]):] = BF16_NAN
        v[b, :, int(sl[b]):] = BF16_NAN
    return q, k, v, sl


def to_pages(cache: np.ndarray, seq_lens, page_tokens: int, seed: int, spare_pages: int = 3):
    """Scatter a contiguous cache [B,Hkv,Lmax,D] into a page pool in a seeded random page order.

    Returns (pages [n_pages,Hkv,page_tokens,D], block_table [B,pages_per_seq] int32).  Unused pool pages and the
    unused tail of each sequence's last page hold NaN bit patterns; table entries beyond a sequence's last page are -1.
    """
    B, Hkv, Lmax, D = cache.shape
    sl = np.asarray(seq_lens, np.int64)
    pps = (Lmax + page_tokens - 1) // page_tokens
    need = [(int(L) + page_tokens - 1) // page_tokens for L in sl]
    n_pages = sum(need) + spare_pages
    order = _rng(seed, 77).permutation(n_pages)
    pages = np.full((n_pages, Hkv, page_tokens, D), BF16_NAN, np.uint16)
    table = np.full((B, pps), -1, np.int32)
    nxt = 0
    for b in range(B):
        for j in range(need[b]):
            pg = int(order[nxt]); nxt += 1
            table[b, j] = pg
            t0, t1 = j * page_tokens, min((j + 1) * page_tokens, int(sl[b]))
            pages[pg, :, :t1 - t0] = cache[b, :, t0:t1]
    return pages, table
