"""Oracle for the search over deployments (paper Section 4.3: initialisation by K-means on the communication
matrices with the number of groups from the elbow of the inertia curve; merge / split / swap mutations; early check;
layer partition by one even -> memory-proportional round; iterate and score by SLO attainment).
TEST INFRASTRUCTURE ONLY: only tests, the smoke check and the CPU-baseline leg of the benchmark may import this file.

The paper names the ingredients and leaves the driver open; this file fixes the following readings (the product's
scheduler states the same ones in its own words, the two share no code):

  random draws   a counter-based generator: draw(seed, c) is output c + 1 of the SplitMix64 sequence started at `seed`
                 (Steele, Lea, Flood 2014); an index below n is draw mod n.  Iteration `it` uses counters 5 it .. 5 it + 4.
  K-means        one point per GPU type that is present, weight = its GPU count (every GPU of a type has the same
                 rows in the communication matrices, so this is K-means over GPUs); features = the type's row of
                 per-hop latencies divided by the largest latency, then its row of per-byte times (1 / bandwidth)
                 divided by the largest per-byte time.  Seeding: the heaviest point, then repeatedly the point farthest
                 from its nearest centre (lowest index on ties).  Lloyd rounds until no assignment changes (at most
                 100); a cluster left empty keeps its centre.
  elbow          W_M = weighted inertia for M = 1 .. n clusters; on the curve (x, y) = ((M-1)/(n-1), W_M / W_1) the
                 elbow is the point farthest below the chord from the first to the last point, the smallest M on
                 ties; M = 1 when n = 1 or W_1 = 0.
  group plan     for S = 1 .. min(max_stages, GPUs in the group, layers): even partition (the first L mod S stages
                 one layer more), solve the layout problem, re-partition proportionally to the memory of the GPUs
                 serving each stage, solve again, keep the cheaper (the even one on ties); over S keep the cheapest
                 (fewest stages on ties).  A stage count whose even partition has no feasible layout is skipped.
  iteration      pick a member of the population, pick merge / split / swap, pick its operand groups (and for swap the
                 GPU type among those the giving group holds), all uniformly by the draws above; an offspring is
                 dropped when an operator does not apply (merge or swap with one group, split of a single GPU), when a
                 new group fails the early memory check, exceeds `max_group_states` layout states, or has no feasible
                 plan.  A surviving offspring joins the population while it has room, else replaces the member of lowest
                 attainment (the oldest of those) unless its own attainment is lower.
  result         the first individual to reach the highest attainment seen."""
from __future__ import annotations

import math
from typing import Dict, List, Sequence, Tuple

from oracle import sched_oracle as sch
from oracle import slo_oracle as slo

_M64 = (1 << 64) - 1


def draw(seed: int, counter: int) -> int:
    z = (seed + (counter + 1) * 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


# ---- initialisation ----------------------------------------------------------------------------------------------
def comm_features(pool) -> Tuple[List[int], List[List[float]], List[float]]:
    """(types present, their feature vectors, their weights)."""
    nt = len(pool["count"])
    present = [k for k in range(nt) if pool["count"][k] > 0]
    a_max = max(pool["pp_alpha"][k][j] for k in present for j in present)
    t_max = max(1.0 / pool["pp_beta"][k][j] for k in present for j in present)
    feats = []
    for k in present:
        row = [pool["pp_alpha"][k][j] / a_max if a_max > 0 else 0.0 for j in present]
        row += [(1.0 / pool["pp_beta"][k][j]) / t_max for j in present]
        feats.append(row)
    return present, feats, [float(pool["count"][k]) for k in present]


def _d2(p: Sequence[float], q: Sequence[float]) -> float:
    return sum((a - b) * (a - b) for a, b in zip(p, q))


def kmeans(points: Sequence[Sequence[float]], weights: Sequence[float], n_clusters: int):
    """Weighted Lloyd iteration with the deterministic seeding described in the header.
    Returns (assignment per point, centres, weighted inertia)."""
    n = len(points)
    assert 1 <= n_clusters <= n
    first = max(range(n), key=lambda i: (weights[i], -i))
    centres = [list(points[first])]
    while len(centres) < n_clusters:
        far = max(range(n), key=lambda i: (min(_d2(points[i], c) for c in centres), -i))
        centres.append(list(points[far]))
    assign = [-1] * n
    for _ in range(100):
        new = [min(range(n_clusters), key=lambda c: (_d2(points[i], centres[c]), c)) for i in range(n)]
        if new == assign:
            break
        assign = new
        for c in range(n_clusters):
            members = [i for i in range(n) if assign[i] == c]
            if not members:
                continue
            w = sum(weights[i] for i in members)
            centres[c] = [sum(weights[i] * points[i][d] for i in members) / w for d in range(len(points[0]))]
    inertia = sum(weights[i] * _d2(points[i], centres[assign[i]]) for i in range(n))
    return assign, centres, inertia


def elbow(inertia: Sequence[float]) -> int:
    """Number of clusters (1-based) at the elbow of the inertia curve W_1 .. W_n."""
    n = len(inertia)
    if n == 1 or inertia[0] <= 0.0:
        return 1
    y_last = inertia[-1] / inertia[0]
    best_m, best_d = 1, 0.0
    for m in range(1, n + 1):
        x = (m - 1) / (n - 1)
        d = (1.0 - (1.0 - y_last) * x) - inertia[m - 1] / inertia[0]
        if d > best_d:
            best_m, best_d = m, d
    return best_m


def initial_groups(pool) -> List[List[int]]:
    """The K-means / elbow initialisation: every cluster of GPU types becomes one pipeline group."""
    nt = len(pool["count"])
    present, feats, weights = comm_features(pool)
    runs = [kmeans(feats, weights, m) for m in range(1, len(present) + 1)]
    m = elbow([r[2] for r in runs])
    assign = runs[m - 1][0]
    groups = []
    for c in range(m):
        tau = [0] * nt
        for i, k in enumerate(present):
            if assign[i] == c:
                tau[k] = pool["count"][k]
        if sum(tau) > 0:
            groups.append(tau)
    return groups


# ---- one group's pipeline ------------------------------------------------------------------------------------------
def layout_states(tau: Sequence[int]) -> int:
    return math.prod(t + 1 for t in tau)


def plan_group(pool, task, tau: Sequence[int], total_layers: int, max_stages: int, degrees=None):
    """(latency, layers per stage, [(type, count)] per stage) of the best pipeline the group can run, or
    (inf, [], []) when it can run none."""
    sub = dict(pool, count=list(tau))
    best = (math.inf, [], [])
    for n_stages in range(1, min(max_stages, sum(tau), total_layers) + 1):
        even = [total_layers // n_stages + (1 if j < total_layers % n_stages else 0) for j in range(n_stages)]
        c1, a1 = sch.best_layout_bruteforce(sub, task, even, degrees)
        if not c1 < math.inf:
            continue
        cand = (c1, even, a1)
        prop = sch.repartition_layers(total_layers, [pool["mem"][k] * n for k, n in a1])
        if prop != even:
            c2, a2 = sch.best_layout_bruteforce(sub, task, prop, degrees)
            if c2 < c1:
                cand = (c2, prop, a2)
        if cand[0] < best[0]:
            best = cand
    return best


# ---- the search ------------------------------------------------------------------------------------------------------
def search(pool, task, total_layers: int, model_bytes: float, max_stages: int, arrival: Sequence[float],
           deadline: float, seed: int, n_iter: int, pop_size: int, degrees=None,
           max_group_states: int = 1 << 14) -> Dict:
    plans: Dict[Tuple[int, ...], tuple] = {}

    def plan(tau):
        key = tuple(tau)
        if key not in plans:
            plans[key] = plan_group(pool, task, tau, total_layers, max_stages, degrees)
        return plans[key]

    def admissible(tau) -> bool:
        return (sum(tau) > 0 and sch.group_can_hold(tau, pool["mem"], model_bytes)
                and layout_states(tau) <= max_group_states and plan(tau)[0] < math.inf)

    def fitness(groups) -> float:
        return slo.attainment(arrival, [[plan(g)[0]] for g in groups], [deadline])

    start = initial_groups(pool)
    if not all(admissible(g) for g in start):
        # reading: an inadmissible start (a cluster too small for the model) falls back to the whole pool as one group
        start = [list(pool["count"])]
        if not admissible(start[0]):
            return {"attainment": math.nan, "groups": [], "history": []}
    population = [(start, fitness(start))]
    best = population[0]
    history = []
    for it in range(n_iter):
        u = [draw(seed, 5 * it + j) for j in range(5)]
        parent = population[u[0] % len(population)][0]
        op = u[1] % 3
        n_g = len(parent)
        child, fresh = None, []
        if op == 0 and n_g >= 2:                                   # merge groups i and j
            i = u[2] % n_g
            j = u[3] % (n_g - 1)
            j += j >= i
            merged = sch.merge(parent[i], parent[j])
            child = [g for x, g in enumerate(parent) if x not in (i, j)] + [merged]
            fresh = [merged]
        elif op == 1:                                              # split group i
            i = u[2] % n_g
            lo, hi = sch.split(parent[i])
            if sum(lo) > 0 and sum(hi) > 0:
                child = [lo if x == i else g for x, g in enumerate(parent)] + [hi]
                fresh = [lo, hi]
        elif op == 2 and n_g >= 2:                                 # one GPU from group j to group i
            i = u[2] % n_g
            j = u[3] % (n_g - 1)
            j += j >= i
            held = [k for k, t in enumerate(parent[j]) if t > 0]
            k = held[u[4] % len(held)]
            gi, gj = sch.swap(parent[i], parent[j], k)
            child = [gi if x == i else gj if x == j else g for x, g in enumerate(parent)]
            fresh = [gi]
            if sum(gj) == 0:
                child = [g for x, g in enumerate(child) if x != j]
            else:
                fresh.append(gj)
        if child is not None and all(admissible(g) for g in fresh):
            f = fitness(child)
            if len(population) < pop_size:
                population.append((child, f))
            else:
                worst = min(range(len(population)), key=lambda x: (population[x][1], x))
                if f >= population[worst][1]:
                    population.pop(worst)
                    population.append((child, f))
            if f > best[1]:
                best = (child, f)
        history.append(best[1])
    groups = [{"tau": list(g), "latency": plan(g)[0], "layers": list(plan(g)[1]), "stages": list(plan(g)[2])}
              for g in best[0]]
    return {"attainment": best[1], "groups": groups, "history": history}
