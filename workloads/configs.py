"""Workload table: the stage shapes this build is measured and parity-tested on.

Holds shapes only -- none of the method's arithmetic.  A stage is one GPU's share of
one pipeline stage of the asymmetric tensor+pipeline engine (paper Section 3): `n_layers`
consecutive decoder layers at tensor-parallel degree `tp_degree`, rank `tp_rank`.
The model served in the paper's evaluation is Llama-2 (70B) (Section 5.1), hence the
70B-shaped entries; the tiny fp32 entry is the case a CPU checker finishes in seconds.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple


@dataclass(frozen=True)
class StageConfig:
    name: str
    dtype: str                 # "f32" | "bf16"
    hidden: int                # H (global)
    n_heads: int               # hq (global query heads)
    n_kv_heads: int            # hkv (global KV heads)
    ffn: int                   # F (global SwiGLU width)
    n_layers: int              # layers in this stage
    tp_degree: int             # t
    tp_ranks: Tuple[int, ...]  # ranks that are run (one entry = solo mode)
    batch: int
    # prompt: fixed length, or (lo, hi) inclusive bounds for ragged lengths, or None when
    # the KV context is synthetic (decode-only workloads)
    prompt_len: Optional[int] = None
    prompt_range: Optional[Tuple[int, int]] = None
    kv_context: Optional[int] = None   # synthetic KV rows present before the first decode
    decode_steps: int = 0
    seed: int = 0
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    vocab: int = 0             # >0: greedy loop through an embedding / LM head of this size

    # ---- derived (local = this rank's share) -------------------------------------
    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads

    @property
    def hq_l(self) -> int:
        return self.n_heads // self.tp_degree

    @property
    def hkv_l(self) -> int:
        return self.n_kv_heads // self.tp_degree

    @property
    def ffn_l(self) -> int:
        return self.ffn // self.tp_degree

    @property
    def group(self) -> int:
        return self.n_heads // self.n_kv_heads

    @property
    def weight_elems_per_layer_rank(self) -> int:
        d = self.head_dim
        qkv = self.hidden * (self.hq_l + 2 * self.hkv_l) * d
        wo = self.hq_l * d * self.hidden
        return qkv + wo + 3 * self.hidden * self.ffn_l

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def kv_bytes_per_pos_layer(self) -> int:
        return 2 * self.hkv_l * self.head_dim * self.elem_bytes

    def scaled(self, **kw) -> "StageConfig":
        return replace(self, **kw)


_L70 = dict(hidden=8192, n_heads=64, n_kv_heads=8, ffn=28672)

CONFIGS = {
    # tiny fp32 stage: both ranks run and their partials are summed (group mode)
    "tiny_f32": StageConfig("tiny_f32", "f32", 512, 8, 2, 1408, 2, 2, (0, 1), batch=1,
                            prompt_len=32, decode_steps=8, seed=0, vocab=1000),
    # 70B shard, TP2 rank 0, 8 layers, batch-1 decode at synthetic context 1024
    "l70_tp2_decode": StageConfig("l70_tp2_decode", "bf16", **_L70, n_layers=8, tp_degree=2,
                                  tp_ranks=(0,), batch=1, kv_context=1024, decode_steps=256,
                                  seed=2),
    # asymmetric shard, TP4 rank 1, 20 layers, prefill 4x512 then 64 decode steps
    "l70_tp4_prefill": StageConfig("l70_tp4_prefill", "bf16", **_L70, n_layers=20, tp_degree=4,
                                   tp_ranks=(1,), batch=4, prompt_len=512, decode_steps=64,
                                   seed=3),
    # TP8 rank 3, 40 layers, batch-16 decode at synthetic context 2048
    "l70_tp8_decode": StageConfig("l70_tp8_decode", "bf16", **_L70, n_layers=40, tp_degree=8,
                                  tp_ranks=(3,), batch=16, kv_context=2048, decode_steps=128,
                                  seed=4),
    # full-width 80-layer stage, 32 ragged prompts then 128 decode steps
    "l70_full": StageConfig("l70_full", "bf16", **_L70, n_layers=80, tp_degree=1,
                            tp_ranks=(0,), batch=32, prompt_range=(128, 4096),
                            decode_steps=128, seed=5),
}

# order in which the benchmark spec lists them
CONFIG_ORDER = ["tiny_f32", "l70_tp2_decode", "l70_tp4_prefill", "l70_tp8_decode", "l70_full"]
