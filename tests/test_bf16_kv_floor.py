"""What a bf16 KV cache alone costs at depth 20 of the TP4 prefill workload -- CPU only, oracle only.

The 70B-shaped stages store K and V in bf16 (the configuration names the type).  This test runs the
oracle twice on the same inputs in float64: once as it stands, once with ONE change -- every K / V row
is rounded to bf16 when it enters the cache -- and measures the distance between the two stage outputs
with the two error metrics the GPU parity tests print.  Nothing else is rounded: projections,
softmax, residual stream and FFN stay float64.  The result is a floor for any implementation with a
bf16 cache on these weights: the rule in the GPU tests (which end-to-end comparisons gate on per-row L2
error and which on max-abs over the row norm) rests on the two assertions at the end.

Shard-shaped weights are drawn directly (same distribution as the workload generator: N(0, 0.02^2)
matrices, gains 1 + 0.02 N(0,1), all rounded to bf16); solo mode of rank r equals an unsharded stage
whose global weights are the shard (pinned in test_oracle_pins), which is how the oracle is built here.
"""
import numpy as np
import torch

from oracle import stage_oracle as so
from tests.helpers import max_abs_over_l2, row_rel_err
from workloads import CONFIGS

CFG = CONFIGS["l70_tp4_prefill"]
ROWS = 48            # prompt rows of the one sequence (cost: the float64 projections of 20 layers)


def _bf16(x: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


class Bf16KVCache(so.KVCache):
    """The oracle's cache with its rows rounded to bf16 on the way in (round to nearest even)."""

    def append(self, layer, seq, k, v):
        super().append(layer, seq, _bf16(k).astype(np.float64), _bf16(v).astype(np.float64))


def _draw_layer(rng, cfg):
    H, d = cfg.hidden, cfg.head_dim
    qw, kw, F = cfg.hq_l * d, cfg.hkv_l * d, cfg.ffn_l

    def mat(*shape):
        return _bf16(0.02 * rng.standard_normal(shape, dtype=np.float32))

    def gain():
        return _bf16(1.0 + 0.02 * rng.standard_normal(H, dtype=np.float32))

    return [gain(), mat(H, qw), mat(H, kw), mat(H, kw), mat(qw, H), gain(), mat(H, F), mat(H, F), mat(F, H)]


def test_bf16_kv_rounding_alone_exceeds_per_row_l2_gate_at_depth_20():
    cfg = CFG
    one = so.OracleStage(cfg.hidden, cfg.hq_l, cfg.hkv_l, cfg.ffn_l, 1, 1, 0, cfg.rms_eps, cfg.rope_theta)
    one.d = cfg.head_dim                      # head_dim belongs to the model, not to hidden / local heads
    rng = np.random.default_rng(20)
    x = _bf16(rng.standard_normal((ROWS, cfg.hidden), dtype=np.float32)).astype(np.float64)
    exact_c = so.KVCache(1, 1, cfg.hkv_l, cfg.head_dim)
    round_c = Bf16KVCache(1, 1, cfg.hkv_l, cfg.head_dim)
    seqs = [0] * ROWS
    h_e, h_r = x.copy(), x.copy()
    trace = []
    for layer in range(cfg.n_layers):
        one.load_layer(0, *_draw_layer(rng, cfg))        # one layer resident at a time
        exact_c.k[0][0] = exact_c.k[0][0][:0]; exact_c.v[0][0] = exact_c.v[0][0][:0]
        round_c.k[0][0] = round_c.k[0][0][:0]; round_c.v[0][0] = round_c.v[0][0][:0]
        h_e = h_e + one.attn_partial(0, exact_c, h_e, seqs)
        h_r = h_r + one.attn_partial(0, round_c, h_r, seqs)
        p_e, p_r = one.ffn_partial(0, h_e), one.ffn_partial(0, h_r)
        trace.append((row_rel_err(h_r, h_e), row_rel_err(p_r, p_e), max_abs_over_l2(h_r, h_e), max_abs_over_l2(p_r, p_e)))
        if layer + 1 < cfg.n_layers:
            h_e, h_r = h_e + p_e, h_r + p_r
    for layer in (0, 3, 9, 19):
        e = trace[layer]
        print(f"bf16 K/V only, after layer {layer}: per-row L2 resid {e[0]:.3e} partial {e[1]:.3e}; "
              f"max-abs / L2 resid {e[2]:.3e} partial {e[3]:.3e}")
    # the perturbation grows with depth on these weights ...
    assert trace[19][1] > trace[3][1] > trace[0][1]
    # ... and at depth 20 the per-row L2 distance of the partial is beyond the 2e-2 gate although only the cache
    # rows were rounded, while the largest element error stays far inside 2e-2 of the row's norm
    assert trace[19][1] > 2e-2
    assert trace[19][2] < 5e-3 and trace[19][3] < 5e-3
