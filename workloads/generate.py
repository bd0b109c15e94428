"""Seeded synthetic inputs shared by the CPU checker's tests and the GPU path's tests.

Only random draws and dtype rounding of *inputs* live here; nothing of the method's
arithmetic.  Everything is returned as fp32 torch tensors.  For a bf16 stage the values are
rounded to bf16 (round-to-nearest-even) first, so the very same numbers can be handed to a
double-precision CPU implementation and, bit-exactly, to a bf16 GPU implementation.

Recipe (all normal draws):
  matrices          ~ N(0, 0.02^2), drawn at GLOBAL (unsharded) shape, [in, out] row-major
  RMSNorm gains     = 1 + 0.02 * N(0, 1)
  hidden inputs     ~ N(0, 1)
  synthetic KV rows ~ N(0, 1)   (decode-only workloads start from such a context)
Every stream's seed is `((cfg.seed * 16 + kind) * 100003 + a) * 100003 + b` with kind
0 = layer weights (a = layer), 1 = prompt lengths, 2 = hidden rows (a = stream id),
3 = synthetic KV (a = layer, b = sequence), 4 = embedding / LM head.  A layer stream draws,
in this fixed order, g_attn, wq, wk, wv, wo, g_ffn, w1, w3, w2.  On `device="cpu"` the stream is numpy's
`default_rng`; on a GPU device it is torch's device generator (much faster for 70B-sized
layers).  The two streams differ, so one test uses one device for both sides.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np
import torch

from .configs import StageConfig

LAYER_TENSOR_ORDER = ("g_attn", "wq", "wk", "wv", "wo", "g_ffn", "w1", "w3", "w2")


def round_to_dtype(x: torch.Tensor, dtype: str) -> torch.Tensor:
    """fp32 tensor whose values are exactly representable in `dtype`."""
    if dtype == "bf16":
        return x.to(torch.bfloat16).to(torch.float32)
    if dtype == "f16":
        return x.to(torch.float16).to(torch.float32)
    if dtype == "f32":
        return x.to(torch.float32)
    raise ValueError(dtype)


class _Stream:
    """Normal draws from one seeded stream on one device."""

    def __init__(self, seed: int, device: str):
        self.device = torch.device(device)
        if self.device.type == "cpu":
            self.rng = np.random.default_rng(seed)
            self.gen = None
        else:
            self.rng = None
            self.gen = torch.Generator(device=self.device)
            self.gen.manual_seed(seed)

    def normal(self, *shape: int) -> torch.Tensor:
        if self.rng is not None:
            return torch.from_numpy(self.rng.standard_normal(shape, dtype=np.float32))
        return torch.randn(*shape, generator=self.gen, device=self.device, dtype=torch.float32)

    def integers(self, lo: int, hi_inclusive: int, n: int) -> List[int]:
        if self.rng is not None:
            return [int(v) for v in self.rng.integers(lo, hi_inclusive + 1, size=n)]
        v = torch.randint(lo, hi_inclusive + 1, (n,), generator=self.gen, device=self.device)
        return [int(t) for t in v.cpu()]


def _seed(cfg: StageConfig, kind: int, a: int = 0, b: int = 0) -> int:
    return ((cfg.seed * 16 + kind) * 100003 + a) * 100003 + b


def layer_shapes(cfg: StageConfig) -> Dict[str, tuple]:
    H, d = cfg.hidden, cfg.head_dim
    return {
        "g_attn": (H,), "wq": (H, cfg.n_heads * d), "wk": (H, cfg.n_kv_heads * d),
        "wv": (H, cfg.n_kv_heads * d), "wo": (cfg.n_heads * d, H), "g_ffn": (H,),
        "w1": (H, cfg.ffn), "w3": (H, cfg.ffn), "w2": (cfg.ffn, H),
    }


def layer_weights(cfg: StageConfig, layer: int, device: str = "cpu") -> Dict[str, torch.Tensor]:
    """Global-shape tensors of one layer (fp32 storage, values representable in cfg.dtype)."""
    s = _Stream(_seed(cfg, 0, layer), device)
    out = {}
    shapes = layer_shapes(cfg)
    for name in LAYER_TENSOR_ORDER:
        z = s.normal(*shapes[name])
        w = 1.0 + 0.02 * z if name.startswith("g_") else 0.02 * z
        out[name] = round_to_dtype(w, cfg.dtype)
    return out


def prompt_lengths(cfg: StageConfig, device: str = "cpu") -> List[int]:
    if cfg.prompt_len is not None:
        return [cfg.prompt_len] * cfg.batch
    if cfg.prompt_range is not None:
        lo, hi = cfg.prompt_range
        return _Stream(_seed(cfg, 1), device).integers(lo, hi, cfg.batch)
    return [0] * cfg.batch


def hidden_rows(cfg: StageConfig, n_rows: int, stream_id: int = 0, device: str = "cpu") -> torch.Tensor:
    """[n_rows, H] stage-input activations ~ N(0,1); stream_id 0 = prompt, 1+k = decode step k."""
    s = _Stream(_seed(cfg, 2, stream_id), device)
    return round_to_dtype(s.normal(n_rows, cfg.hidden), cfg.dtype)


def synthetic_kv(cfg: StageConfig, layer: int, seq: int, n: int, device: str = "cpu"):
    """(K, V), each [n, hkv_l, d] ~ N(0,1): a stand-in context for decode-only workloads."""
    s = _Stream(_seed(cfg, 3, layer, seq), device)
    k = round_to_dtype(s.normal(n, cfg.hkv_l, cfg.head_dim), cfg.dtype)
    v = round_to_dtype(s.normal(n, cfg.hkv_l, cfg.head_dim), cfg.dtype)
    return k, v


def head_weights(cfg: StageConfig, device: str = "cpu") -> Dict[str, torch.Tensor]:
    """Embedding E [vocab,H], final-norm gain [H], untied LM head [H,vocab] for the greedy loop."""
    assert cfg.vocab > 0
    s = _Stream(_seed(cfg, 4), device)
    emb = round_to_dtype(0.02 * s.normal(cfg.vocab, cfg.hidden), cfg.dtype)
    g = round_to_dtype(1.0 + 0.02 * s.normal(cfg.hidden), cfg.dtype)
    lm = round_to_dtype(0.02 * s.normal(cfg.hidden, cfg.vocab), cfg.dtype)
    return {"embedding": emb, "g_final": g, "w_lm": lm}
