"""Per-layer driver for a decode step over a stack of attention layers (host-side glue only).

The paper routes every layer except the first two, whose heads behave atypically (Appendix B);
the library itself has no notion of a layer, so this helper owns one ``sr_route_params`` per layer
(routing switched off below ``first_routed_layer``), one shared workspace, and enqueues the layers
back to back on the current stream.  Everything it calls is allocation-free after construction, so
``step`` can be captured into a HIP graph.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

from . import binding


class LayerStack:
    def __init__(self, k_caches: Sequence, v_caches: Sequence, seq_lens, n_q_heads: int, *,
                 first_routed_layer: int = 2, tau_coef=(0.0, 0.0, 0.0, 0.55), len_norm: float = 0.0,
                 sm_scale: float = 0.0, num_splits: int = 0):
        import torch
        assert len(k_caches) == len(v_caches) and len(k_caches) > 0
        self.k, self.v, self.seq_lens = list(k_caches), list(v_caches), seq_lens
        B, Hkv, Lmax, D = self.k[0].shape
        self.shape = (B, n_q_heads, Hkv, Lmax, D)
        self.first_routed_layer = int(first_routed_layer)
        dev = self.k[0].device
        probe = binding.make_route_params(B, n_q_heads, Hkv, Lmax, head_dim=D, num_splits=num_splits)
        self.plan = binding.sinkrouter_plan(probe)
        # the layers run one after another on one stream, so they can share the workspace
        self.workspace = torch.empty((self.plan.workspace_bytes,), dtype=torch.uint8, device=dev)
        self.params: List[binding.RouteParams] = []
        for layer in range(len(self.k)):
            self.params.append(binding.make_route_params(
                B, n_q_heads, Hkv, Lmax, head_dim=D, num_splits=num_splits, sm_scale=sm_scale,
                routing_enabled=layer >= self.first_routed_layer, tau_coef=tau_coef, len_norm=len_norm,
                workspace=self.workspace))
        self.out = [torch.empty((B, n_q_heads, D), dtype=torch.int16, device=dev) for _ in self.k]
        self.mask = [torch.empty((B, Hkv), dtype=torch.uint8, device=dev) for _ in self.k]

    def step(self, queries: Sequence, layers: Optional[Sequence[int]] = None) -> None:
        """Enqueue the decode step of every layer (or of ``layers``); queries[l] is layer l's q [B,Hq,D]."""
        for layer in (range(len(self.k)) if layers is None else layers):
            binding.sinkrouter_decode(queries[layer], self.k[layer], self.v[layer], self.seq_lens,
                                      self.params[layer], self.out[layer], self.mask[layer])
