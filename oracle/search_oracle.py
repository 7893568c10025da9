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


def algorithm1(measure: Measure, n_m: int, n_d: int, L: float,
               P: float = float("inf")) -> Tuple[Optional[Point], List[Point]]:
    """Returns (configuration or None if even the origin breaks the bounds, path)."""
    cur = (0, 0)                                            # Initialize batch size, num of threads
    qps_prev, lat_prev, pow_prev = measure(*cur)
    if not (lat_prev < L and pow_prev < P):
        return None, [cur]
    path = [cur]
    while True:
        mi, di = cur
        candidates = [(mi, di + 1), (mi + 1, di), (mi + 1, di + 1)]   # three candidates
        grad_qps, valid = [], []
        for c in candidates:
            if c[0] >= n_m or c[1] >= n_d:
                grad_qps.append(float("-inf"))
                valid.append(False)
                continue
            qps_t, lat_t, pow_t = measure(*c)
            grad_qps.append(qps_t - qps_prev)               # nabla QPS = QPS_t - QPS_{t-1}
            valid.append(lat_t < L and pow_t < P)           # nabla Latency decides through L
        best, best_gain = None, 0.0
        for c, g, ok in zip(candidates, grad_qps, valid):
            if ok and g > best_gain:
                best, best_gain = c, g
        if best is None:                                    # no throughput increase within bounds
            return cur, path
        cur = best                                          # update to Configuration(max(Candidate))
        qps_prev = qps_prev + best_gain
        path.append(cur)


def exhaustive(measure: Measure, n_m: int, n_d: int, L: float,
               P: float = float("inf")) -> Tuple[Optional[Point], float]:
    best, best_qps = None, float("-inf")
    for mi in range(n_m):
        for di in range(n_d):
            qps, lat, pw = measure(mi, di)
            if lat < L and pw < P and qps > best_qps:
                best, best_qps = (mi, di), qps
    return best, best_qps
