"""Shared helpers for the GPU parity tests: build both sides from one set of seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

from workloads import generate

ORDER = generate.LAYER_TENSOR_ORDER
# max per-row ||gpu - ref|| / ||ref||: the benchmark spec's tolerances for f32 and bf16; fp16 takes the bf16 gate scaled by the
# ratio of the unit roundoffs (2^-11 / 2^-9)
TOL = {"f32": 1e-4, "bf16": 2e-2, "f16": 5e-3}


def row_rel_err(gpu, ref) -> float:
    """max over rows of ||gpu_i - ref_i||_2 / ||ref_i||_2 (stricter than a whole-tensor norm)."""
    g = np.asarray(gpu, dtype=np.float64).reshape(-1, np.asarray(ref).shape[-1])
    r = np.asarray(ref, dtype=np.float64).reshape(g.shape)
    num = np.linalg.norm(g - r, axis=1)
    den = np.linalg.norm(r, axis=1)
    return float(np.max(num / den))


def max_abs_over_l2(gpu, ref) -> float:
    """max over rows of max_c |gpu - ref| / ||ref_row||_2: the largest elementwise error measured against
    the L2 norm of the output row (the literal form of "max relative error, relative to the output's L2
    norm").  Used as the end-to-end gate only where bf16 storage makes the per-row L2 gate unattainable."""
    g = np.asarray(gpu, dtype=np.float64).reshape(-1, np.asarray(ref).shape[-1])
    r = np.asarray(ref, dtype=np.float64).reshape(g.shape)
    return float(np.max(np.max(np.abs(g - r), axis=1) / np.linalg.norm(r, axis=1)))


def check(label: str, gpu, ref, tol: float, per_row_l2: bool = True):
    """THE gate of the GPU parity tests.  Prints both error metrics of one comparison and asserts
      G1  max_abs_over_l2 < tol   always (the stated tolerance: largest error relative to the output row's L2 norm);
      G2  row_rel_err     < tol   as well, unless per_row_l2=False.
    per_row_l2=False is passed by exactly one family of comparisons: the END-TO-END outputs of the 20-layer
    prefill workload, where rounding K and V to the bf16 the cache stores -- and nothing else -- already puts G2
    beyond 2e-2 (tests/test_bf16_kv_floor.py, CPU, oracle only); there every layer is compared on its own,
    fed the oracle's residual stream, with G2 on.  Returns (G2, G1)."""
    e2, e1 = row_rel_err(gpu, ref), max_abs_over_l2(gpu, ref)
    print(f"{label}: per-row L2 err {e2:.3e}, max-abs / row L2 {e1:.3e}"
          + ("" if per_row_l2 else "  [gate: max-abs / row L2 only]"), flush=True)
    assert e1 < tol, f"{label}: max-abs / row L2 {e1:.3e} >= {tol}"
    if per_row_l2:
        assert e2 < tol, f"{label}: per-row L2 err {e2:.3e} >= {tol}"
    return e2, e1


def torch_dtype(cfg):
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[cfg.dtype]


def make_oracle(cfg, rank, weights, n_layers=None):
    from oracle import stage_oracle as so
    L = cfg.n_layers if n_layers is None else n_layers
    st = so.OracleStage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, L, cfg.tp_degree, rank,
                        cfg.rms_eps, cfg.rope_theta)
    for l in range(L):
        st.load_layer(l, *[weights[l][k] for k in ORDER])
    return st


def make_gpu_stage(cfg, rank, weights, n_layers=None):
    import paper_2311_11514_amd as hx
    L = cfg.n_layers if n_layers is None else n_layers
    st = hx.Stage(cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.ffn, L, cfg.tp_degree, rank, cfg.dtype,
                  cfg.rms_eps, cfg.rope_theta)
    for l in range(L):
        st.load_layer(l, *[weights[l][k] for k in ORDER])
    return st


def to_dev(x, cfg):
    return x.to(device="cuda", dtype=torch_dtype(cfg)).contiguous()


def gpu_prefill(st, kv, cfg, x, seq_lens):
    xin = to_dev(x, cfg)
    outp = torch.empty_like(xin)
    outr = torch.empty_like(xin)
    st.prefill(kv, xin, seq_lens, outp, outr)
    torch.cuda.synchronize()
    return outp.float().cpu().numpy(), outr.float().cpu().numpy()


def gpu_decode(st, kv, cfg, step, x):
    xin = to_dev(x, cfg)
    outp = torch.empty_like(xin)
    outr = torch.empty_like(xin)
    st.decode(kv, step, xin, outp, outr)
    torch.cuda.synchronize()
    return outp.float().cpu().numpy(), outr.float().cpu().numpy()
