"""Oracle for the SLO attainment of a deployment under a request trace (paper Section 5.1, "SLO attainment": the share
of requests finished within the deadline, requests arriving as a Poisson process; Section 4.3, "Put it together":
the search scores a deployment by its expected attainment).  TEST INFRASTRUCTURE ONLY: only tests, the smoke check
and the CPU-baseline leg of the benchmark may import this file; the product never does.

The paper takes its task simulator from another system and gives no listing of it, so the queueing discipline is
this build's reading:
  * a deployment is a set of independent model replicas (pipeline groups); replica r needs latency[r][c] seconds for
    a request of class c (the end-to-end cost of Section 4.2 for that group);
  * requests are taken in arrival order (first come, first served) and never dropped or pre-empted;
  * a replica serves one request at a time;
  * a request goes to the replica on which it would FINISH earliest, given what is already queued there
    (start = max(arrival, time the replica becomes free)); the lowest replica index wins a tie;
  * attainment = #{k : finish_k <= arrival_k + deadline[class_k]} / #requests (in this form a request that never
    waits meets a deadline equal to its latency whatever the rounding of the sums).
Plain Python loops, float64."""
from __future__ import annotations

from typing import List, Optional, Sequence


def simulate(arrival: Sequence[float], latency: Sequence[Sequence[float]],
             cls: Optional[Sequence[int]] = None) -> List[float]:
    """Finish time of every request.  arrival: non-decreasing times >= 0; latency[r][c] > 0."""
    n_rep = len(latency)
    assert n_rep >= 1
    free_at = [0.0] * n_rep                      # replica r has nothing queued from this time on
    finish = []
    last = 0.0
    for k, a in enumerate(arrival):
        assert a >= last, "arrivals must be sorted"
        last = a
        c = 0 if cls is None else cls[k]
        best_r, best_f = -1, 0.0
        for r in range(n_rep):
            start = a if a > free_at[r] else free_at[r]
            f = start + latency[r][c]
            if best_r < 0 or f < best_f:
                best_r, best_f = r, f
        free_at[best_r] = best_f
        finish.append(best_f)
    return finish


def attainment(arrival: Sequence[float], latency: Sequence[Sequence[float]], deadline: Sequence[float],
               cls: Optional[Sequence[int]] = None) -> float:
    """Share of the requests finished by their arrival time plus the deadline of their class."""
    assert len(arrival) >= 1
    finish = simulate(arrival, latency, cls)
    ok = 0
    for k, (a, f) in enumerate(zip(arrival, finish)):
        c = 0 if cls is None else cls[k]
        if f <= a + deadline[c]:
            ok += 1
    return ok / len(arrival)
