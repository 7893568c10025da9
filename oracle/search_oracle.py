"""Oracle of the accelerator-side parallelism search.  TEST INFRASTRUCTURE ONLY.

Two plain statements, used to check the scheduler of the device package (which
imports nothing from here):

* `algorithm1` - the gradient-based search of Algorithm 1 restricted to the
  space the paper gives an accelerator, P_sp(M+D): m co-located inference
  threads (model co-location) and batch size d (query fusion), Sec. II-B and
  Sec. IV-A.  Op-parallelism exists on CPUs only, so its outer loop has one
  pass.  Steps in the paper's order: start at minimal co-location and minimal
  batch size; the three candidates are (d up), (m up), (d and m up); gradients
  of tail latency and throughput are taken against the current point; only
  candidates within the SLA latency L (and power P, when measured) are valid;
  move to the valid candidate with the largest throughput gain; stop when no
  valid candidate gains throughput.
* `exhaustive` - the definition of what the search is after: the highest
  throughput among all grid points whose tail latency (and power) is in bound.

The measurement is passed in as a function (m_index, d_index) -> (qps,
latency, power); the oracle holds no measurement of its own.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Tuple

Point = Tuple[int, int]                       # (index into m_values, index into d_values)
Measure = Callable[[int, int], Tuple[float, float, float]]


def _moves(p: Point, n_m: int, n_d: int) -> List[Point]:
    """Grid points one step away in the directions the search may take: a larger
    batch, one more co-located instance, or both."""
    mi, di = p
    steps = [(mi, di + 1), (mi + 1, di), (mi + 1, di + 1)]
    return [q for q in steps if q[0] < n_m and q[1] < n_d]


def algorithm1(measure: Measure, n_m: int, n_d: int, L: float,
               P: float = float("inf")) -> Tuple[Optional[Point], List[Point]]:
    """Hill climb over the (instances, batch) grid from its smallest corner
    (Algorithm 1, Sec. IV-A, restricted to P_sp(M+D)).  Returns (end point, or
    None when even the starting corner is out of bounds; points visited)."""
    def admissible(lat: float, power: float) -> bool:
        return lat < L and power < P

    here: Point = (0, 0)
    here_qps, lat0, pow0 = measure(*here)
    visited = [here]
    if not admissible(lat0, pow0):
        return None, visited
    while True:
        # throughput gained by each admissible move, measured against the point we stand on
        gains = {}
        for q in _moves(here, n_m, n_d):
            qps, lat, power = measure(*q)
            if admissible(lat, power):
                gains[q] = qps - here_qps
        # the first of the best: ties keep the order batch, instances, both
        winner = max(gains, key=gains.get, default=None)
        if winner is None or gains[winner] <= 0.0:
            return here, visited
        here_qps += gains[winner]
        here = winner
        visited.append(here)


def exhaustive(measure: Measure, n_m: int, n_d: int, L: float,
               P: float = float("inf")) -> Tuple[Optional[Point], float]:
    best, best_qps = None, float("-inf")
    for mi in range(n_m):
        for di in range(n_d):
            qps, lat, pw = measure(mi, di)
            if lat < L and pw < P and qps > best_qps:
                best, best_qps = (mi, di), qps
    return best, best_qps
