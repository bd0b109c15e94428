"""Oracle for the paper's pipeline-layout optimisation (Section 4.2, Eq. "end-to-end cost" and the DP of Algorithm 1)
and for the search's mutation operators (Section 4.3).  TEST INFRASTRUCTURE ONLY.

The layout problem: a pipeline group holds #_k GPUs of each of N_T types; a layer partition l_1 .. l_S is given;
every stage j runs on tau_k GPUs of ONE type k (the paper's heuristic: a tensor-parallel group uses the same type of
GPU on the same machine).  The oracle is the definition written out: enumerate every assignment of (type, count) to
the stages that the group can supply, evaluate the end-to-end cost with the cost-model oracle, keep the minimum.
Exponential -- small cases only.  GPUs may stay unused (reading: the DP's answer is the best entry of its last row)."""
from __future__ import annotations

import itertools
import math
from typing import List, Sequence, Tuple

from oracle import cost_oracle as co


def stage_cost(pool, task, layers, k, n) -> float:
    """Computation + tensor-parallel traffic of one stage of `layers` layers on n GPUs of type k; +inf when the stage
    does not fit the type's memory (Eq. 6)."""
    H, pf, B, b, s_in, s_out = task
    if co.mem(H, B, b, s_in, s_out, layers, n, pf) > pool["mem"][k]:
        return math.inf
    comp = co.comp(H, B, b, s_in, s_out, layers, [pool["m"][k]] * n, [pool["c"][k]] * n, pf)
    al = [[pool["tp_alpha"][k]] * n for _ in range(n)]
    be = [[pool["tp_beta"][k]] * n for _ in range(n)]
    return comp + co.comm_tp(H, B, b, s_in, s_out, layers, al, be)


def hop_cost(pool, task, k_from, k_to) -> float:
    H, pf, B, b, s_in, s_out = task
    return co.comm_pp(H, B, b, s_in, s_out, [[pool["pp_alpha"][k_from][k_to]]], [[pool["pp_beta"][k_from][k_to]]])


def best_layout_bruteforce(pool, task, layers: Sequence[int], degrees=None) -> Tuple[float, List[Tuple[int, int]]]:
    """min over all feasible assignments of sum_j stage_cost + sum_{j<S} hop_cost; returns (cost, [(type, count)])."""
    n_types = len(pool["count"])
    options = [(k, n) for k in range(n_types) for n in range(1, pool["count"][k] + 1) if degrees is None or n in degrees]
    best, best_asg = math.inf, []
    for asg in itertools.product(options, repeat=len(layers)):
        used = [0] * n_types
        for k, n in asg:
            used[k] += n
        if any(used[k] > pool["count"][k] for k in range(n_types)):
            continue
        total = sum(stage_cost(pool, task, layers[j], k, n) for j, (k, n) in enumerate(asg))
        total += sum(hop_cost(pool, task, asg[j][0], asg[j + 1][0]) for j in range(len(layers) - 1))
        if total < best:
            best, best_asg = total, list(asg)
    return best, best_asg


# ---- mutation operators of the search (Section 4.3), on the vector representation tau of a group ------------------
def merge(t1: Sequence[int], t2: Sequence[int]) -> List[int]:
    return [a + b for a, b in zip(t1, t2)]


def split(t: Sequence[int]) -> Tuple[List[int], List[int]]:
    return [a // 2 for a in t], [a - a // 2 for a in t]


def swap(t1: Sequence[int], t2: Sequence[int], k: int) -> Tuple[List[int], List[int]]:
    """Move one GPU of type k from the second group to the first."""
    assert t2[k] >= 1
    a, b = list(t1), list(t2)
    a[k] += 1
    b[k] -= 1
    return a, b


def group_can_hold(t: Sequence[int], mem: Sequence[float], model_bytes: float) -> bool:
    """Early check on an offspring (Section 4.3): a group whose total device memory cannot even hold one copy of the
    model parameters is discarded before the layout problem is solved for it."""
    return sum(n * m for n, m in zip(t, mem)) >= model_bytes


def repartition_layers(total_layers: int, stage_mem: Sequence[float]) -> List[int]:
    """Layer partition proportional to the total memory of the GPU set serving each stage (Section 4.3, "Determine the
    pipeline partitions"); reading: every stage keeps at least one layer, shares are floored and the remainder goes
    to the stages with the largest fractional parts, first stage first on ties."""
    S = len(stage_mem)
    assert total_layers >= S
    tot = float(sum(stage_mem))
    extra = total_layers - S
    ideal = [extra * m / tot for m in stage_mem]
    out = [1 + int(math.floor(x)) for x in ideal]
    rest = total_layers - sum(out)
    order = sorted(range(S), key=lambda j: (-(ideal[j] - math.floor(ideal[j])), j))
    for j in order[:rest]:
        out[j] += 1
    return out
