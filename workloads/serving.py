"""Seeded synthetic inputs of the scheduler's search: GPU pools and request traces (inputs only, none of the method's
arithmetic).

Pools are dictionaries in the vector representation of the paper's cost model: per GPU type k the count, memory
bandwidth m [B/s], peak rate c [FLOP/s], memory mem [B], the link inside a tensor-parallel group (tp_alpha [s],
tp_beta [B/s]) and, per ordered pair of types, the link of a pipeline hop (pp_alpha, pp_beta).

`hetero_pool` has the SHAPE of the paper's rented pools (Section 5.1: full-price = 58 GPUs of four models in four
regions, half-price = its first three entries); a type here is one GPU model in one region.  The device figures are
nominal datasheet values, the link figures are synthetic (same machine / same region / across regions): the paper
does not print its measured matrices.  `tiny_pool` draws small random pools for the checks that enumerate.

`poisson_arrivals` draws a request trace: exponential inter-arrival times at the given rate (Section 5.1)."""
from __future__ import annotations

from typing import Dict, List

import numpy as np

# (region, model, count)
_FULL_PRICE = [("iceland", "3090ti", 16), ("norway", "3090ti", 6), ("nevada", "a5000", 8),
               ("illinois", "a6000", 16), ("illinois", "a5000", 8), ("illinois", "a40", 4)]
# nominal: memory bandwidth [B/s], dense 16-bit matrix rate [FLOP/s], memory [B]
_DEVICE = {"3090ti": (1008e9, 160e12, 24e9), "a5000": (768e9, 111e12, 24e9),
           "a6000": (768e9, 155e12, 48e9), "a40": (696e9, 150e12, 48e9)}


def hetero_pool(kind: str = "full_price") -> Dict:
    rows = _FULL_PRICE if kind == "full_price" else _FULL_PRICE[:3]
    assert kind in ("full_price", "half_price")
    nt = len(rows)
    pool = {"count": [r[2] for r in rows], "m": [_DEVICE[r[1]][0] for r in rows], "c": [_DEVICE[r[1]][1] for r in rows],
            "mem": [_DEVICE[r[1]][2] for r in rows],
            "tp_alpha": [12e-6] * nt, "tp_beta": [20e9] * nt,                   # PCIe inside a machine
            "pp_alpha": [[0.0] * nt for _ in range(nt)], "pp_beta": [[0.0] * nt for _ in range(nt)],
            "names": [f"{r[0]}/{r[1]}" for r in rows]}
    for a in range(nt):
        for b in range(nt):
            if a == b:
                al, be = 30e-6, 10e9                                            # same type: same or neighbouring machine
            elif rows[a][0] == rows[b][0]:
                al, be = 0.5e-3, 1.2e9                                          # same region
            else:
                al, be = 40e-3 + 5e-3 * abs(a - b), 0.12e9                      # across regions
            pool["pp_alpha"][a][b], pool["pp_beta"][a][b] = al, be
    return pool


def tiny_pool(seed: int, n_types: int, max_count: int = 3, two_regions: bool = True) -> Dict:
    """Small random pool with pairwise different device figures (no exact ties between layouts)."""
    rng = np.random.default_rng(1000 + seed)
    region = [k % 2 if two_regions else 0 for k in range(n_types)]
    pool = {"count": [int(rng.integers(1, max_count + 1)) for _ in range(n_types)],
            "m": list(rng.uniform(0.6e12, 3e12, n_types)), "c": list(rng.uniform(100e12, 900e12, n_types)),
            "mem": [float(x) for x in rng.choice([24e9, 48e9, 80e9], n_types)],
            "tp_alpha": list(rng.uniform(5e-6, 20e-6, n_types)), "tp_beta": list(rng.uniform(15e9, 200e9, n_types)),
            "pp_alpha": [[0.0] * n_types for _ in range(n_types)], "pp_beta": [[0.0] * n_types for _ in range(n_types)]}
    for a in range(n_types):
        for b in range(n_types):
            near = region[a] == region[b]
            pool["pp_alpha"][a][b] = float(rng.uniform(20e-6, 60e-6) if near else rng.uniform(20e-3, 60e-3))
            pool["pp_beta"][a][b] = float(rng.uniform(5e9, 20e9) if near else rng.uniform(0.05e9, 0.3e9))
    return pool


def poisson_arrivals(rate: float, n: int, seed: int) -> List[float]:
    """n arrival times of a Poisson process of `rate` requests per second, starting after time 0."""
    rng = np.random.default_rng(2000 + seed)
    return [float(t) for t in np.cumsum(rng.exponential(1.0 / rate, n))]
