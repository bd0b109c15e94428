"""Oracle for the paper's inference cost model (Table 1; Appendix "Modeling the Generative Inference Cost",
Eqs. 3-6).  TEST INFRASTRUCTURE ONLY: plain float64 Python written from the formulas, in the paper's notation;
the product (the host functions hexgen_cost_* of the library) shares no code with it.

Notation: H hidden size; B_type bytes per element; task t = (b, s_in, s_out); a stage = l layers on the device set d;
every device has a memory bandwidth m_d (bytes/s) and a peak rate c_d (flop/s); alpha / beta are the latency (s) and
bandwidth (bytes/s) of a link.  `params_factor` is the number of parameters of one layer in units of H^2: the
paper's layer (four H x H attention matrices, one H x 4H and one 4H x H FFN matrix) has 12."""
from __future__ import annotations

from typing import Sequence


def comp_prefill(H, B_type, b, s_in, s_out, l, m, c, params_factor=12.0) -> float:
    """Prefill share of Eq. 3: the matrix-multiplication term for the s_in prompt positions,
    max_d( 2 * params * b * s_in / (|d| c_d) ) * l  (24 b s_in H^2 / (|d| c_d) for the paper's layer)."""
    n = len(c)
    return max(2.0 * params_factor * H * H * b * s_in / (n * cd) for cd in c) * l


def comp_decode(H, B_type, b, s_in, s_out, l, m, c, params_factor=12.0) -> float:
    """Decode share of Eq. 3: per generated token one scan of the stage's parameters through the slowest device's
    memory plus the matrix multiplications of b rows, times s_out tokens."""
    n = len(c)
    scan = max(params_factor * H * H * B_type / (n * md) for md in m)
    flops = max(2.0 * params_factor * H * H * b / (n * cd) for cd in c)
    return (scan + flops) * l * s_out


def comp(H, B_type, b, s_in, s_out, l, m, c, params_factor=12.0) -> float:
    """Eq. 3 as printed: max_d(12 H^2 B s_out / (|d| m_d)) l + max_d(24 b (s_in + s_out) H^2 / (|d| c_d)) l."""
    n = len(c)
    scan = max(params_factor * H * H * B_type * s_out / (n * md) for md in m)
    flops = max(2.0 * params_factor * b * (s_in + s_out) * H * H / (n * cd) for cd in c)
    return scan * l + flops * l


def comm_tp(H, B_type, b, s_in, s_out, l, alpha: Sequence[Sequence[float]], beta: Sequence[Sequence[float]]) -> float:
    """Eq. 4: two all-reduces per layer, each a reduce-scatter and an all-gather superstep (4 supersteps per layer);
    in a superstep device d exchanges a 1/|d| chunk with every other device, the superstep costs the slowest
    device's sum; prefill moves b s_in H B bytes per all-reduce, every decode step b H B."""
    n = len(alpha)
    if n == 1:
        return 0.0
    def superstep(nbytes):
        return max(sum(alpha[d][e] + nbytes / (n * beta[d][e]) for e in range(n) if e != d) for d in range(n))
    return superstep(b * s_in * H * B_type) * 4 * l + superstep(b * H * B_type) * 4 * s_out * l


def comm_pp(H, B_type, b, s_in, s_out, alpha: Sequence[Sequence[float]], beta: Sequence[Sequence[float]]) -> float:
    """Eq. 5: the activation crosses the fastest link between the two stages (alpha[d][d'], beta[d][d'] for d in stage
    j, d' in stage j + 1): once for the prompt, once per generated token."""
    pairs = [(alpha[d][e], beta[d][e]) for d in range(len(alpha)) for e in range(len(alpha[d]))]
    prefill = min(a + b * s_in * H * B_type / bw for a, bw in pairs)
    step = min(a + b * H * B_type / bw for a, bw in pairs)
    return prefill + step * s_out


def mem(H, B_type, b, s_in, s_out, l, n_dev, params_factor=12.0) -> float:
    """Eq. 6: parameters and K / V of the stage's layers, both split over the devices, plus four reusable
    activation buffers of b (s_in + s_out) H elements."""
    s = s_in + s_out
    return (params_factor * H * H * B_type / n_dev + 2.0 * b * s * H * B_type / n_dev) * l + 4.0 * b * s * H * B_type
