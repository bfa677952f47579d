"""Seeded synthetic VLM-shaped inputs for the KVCapsule hot path.

This module holds NO arithmetic of the method: it only draws random tensors with the
shapes and value laws of the benchmark workloads and rounds them once to the storage
type.  It serves both the HIP library (tests, bench) and the CPU oracle (tests), which
otherwise share nothing.  The compressed length m is an argument, never computed here.

Value laws: K, V, q, new-token k, v ~ N(0,1); each K channel is multiplied by a scale
drawn from U(0.5, 4) per (layer, KV head); text K/V follow the same law as vision K/V.
Parameters per layer: M = sorted random m-subset of {0..n-1}; theta[h] ~ N(0, 1/m)
(fan-in of the map m -> n); U[h] ~ N(0, 1/n) (fan-in of the map n -> m); mu[h] ~ N(0, 1/d).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

import torch

BASE_SEED = 20260516


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # position in the benchmark's list of configurations
    layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f32" | "bf16"
    n_img_tokens: int     # n
    n_images: int         # I
    compression: float    # c
    text_len: int         # text rows in the cache before the first decode step
    steps: int            # decode steps of the run

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def text_cap(self) -> int:
        return self.text_len + self.steps

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {w.name: w for w in [
    Workload("tiny", 0, 1, 1, 8, 2, 64, "f32", 576, 1, 0.6, 64, 1),
    Workload("llava15", 1, 1, 8, 32, 32, 128, "bf16", 576, 1, 0.6, 128, 32),
    Workload("llavanext", 2, 32, 16, 32, 32, 128, "bf16", 576, 5, 0.6, 256, 64),
    Workload("qwen2vl", 3, 28, 4, 28, 4, 128, "bf16", 1024, 8, 0.6, 512, 64),
    Workload("video", 4, 28, 8, 28, 4, 128, "bf16", 256, 64, 0.6, 1024, 128),
]}


def seed_for(w: Workload, layer: int, stream: int = 0) -> int:
    return BASE_SEED + 1000 * w.index + layer + 100000 * stream


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_params(w: Workload, m: int, layer: int = 0, device="cpu"):
    """-> dict(key_idx int32 [m], theta [H_kv,m,n], U [H_kv,m,n], mu [H_kv,d]) in w's dtype."""
    g = _gen(seed_for(w, layer, 1), device)
    n, H, d = w.n_img_tokens, w.n_kv_heads, w.head_dim
    perm = torch.randperm(n, generator=g, device=device)
    key_idx = torch.sort(perm[:m]).values.to(torch.int32)
    theta = torch.randn((H, m, n), generator=g, device=device) * (1.0 / m) ** 0.5
    U = torch.randn((H, m, n), generator=g, device=device) * (1.0 / n) ** 0.5
    mu = torch.randn((H, d), generator=g, device=device) * (1.0 / d) ** 0.5
    dt = w.torch_dtype
    return dict(key_idx=key_idx.contiguous(), theta=theta.to(dt).contiguous(),
                U=U.to(dt).contiguous(), mu=mu.to(dt).contiguous())


def channel_scale(w: Workload, layer: int, device="cpu") -> torch.Tensor:
    """[H_kv, d] multipliers of the K channels, U(0.5, 4)."""
    g = _gen(seed_for(w, layer, 2), device)
    return 0.5 + 3.5 * torch.rand((w.n_kv_heads, w.head_dim), generator=g, device=device)


def make_prefill_kv(w: Workload, layer: int = 0, pre_text: int = 0, post_text: int = 0, device="cpu"):
    """Prefill K, V [B, H_kv, S, d] with S = pre_text + I*n + post_text; the vision span
    starts at row pre_text.  Returned in w's dtype."""
    g = _gen(seed_for(w, layer, 3), device)
    S = pre_text + w.n_images * w.n_img_tokens + post_text
    shp = (w.batch, w.n_kv_heads, S, w.head_dim)
    K = torch.randn(shp, generator=g, device=device)
    K *= channel_scale(w, layer, device)[None, :, None, :]
    V = torch.randn(shp, generator=g, device=device)
    return K.to(w.torch_dtype).contiguous(), V.to(w.torch_dtype).contiguous()


def make_text_cache(w: Workload, layer: int = 0, device="cpu", cap: int | None = None):
    """Text K, V caches [B, H_kv, cap, d] with every row drawn (callers treat the first
    text_len rows as valid); same value law as the vision K/V."""
    g = _gen(seed_for(w, layer, 4), device)
    cap = w.text_cap if cap is None else cap
    shp = (w.batch, w.n_kv_heads, cap, w.head_dim)
    K = torch.randn(shp, generator=g, device=device)
    K *= channel_scale(w, layer, device)[None, :, None, :]
    V = torch.randn(shp, generator=g, device=device)
    return K.to(w.torch_dtype).contiguous(), V.to(w.torch_dtype).contiguous()


def make_step_inputs(w: Workload, layer: int, step: int, device="cpu"):
    """-> q [B, H_q, d], k_new, v_new [B, H_kv, d] for one decode step."""
    g = _gen(seed_for(w, layer, 5) + 7919 * (step + 1), device)
    q = torch.randn((w.batch, w.n_q_heads, w.head_dim), generator=g, device=device)
    k = torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=g, device=device)
    k *= channel_scale(w, layer, device)[None, :, :]
    v = torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=g, device=device)
    dt = w.torch_dtype
    return q.to(dt).contiguous(), k.to(dt).contiguous(), v.to(dt).contiguous()
