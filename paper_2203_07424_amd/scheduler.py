"""Accelerator-side task scheduling: which batch size and how many co-located
model instances give the highest latency-bounded throughput.

The paper's task scheduler explores, per server, model-parallelism (co-located
inference threads, m), data-parallelism (batch size, d) and, on CPUs only,
op-parallelism (Sec. II-B); on an accelerator the space is P_sp(M+D), found
convex in throughput and tail latency, and Algorithm 1 walks it by gradients
(Sec. IV-A).  `search` is that walk; `measure_point` measures one (m, d) point
on the GPU with the forward pass of this package, closed loop: every round puts
one batch on each of the m instances' streams and waits for all of them, so
the round time is the tail latency of its batches and m * d / round time the
throughput.
"""
from __future__ import annotations

import time
from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Sequence, Tuple


@dataclass
class Measurement:
    qps: float            # samples per second
    latency_ms: float     # tail (p99) latency of a batch
    power_w: float = 0.0  # not measured on this machine; kept for the power bound


@dataclass
class SearchResult:
    instances: Optional[int]
    batch: Optional[int]
    measurement: Optional[Measurement]
    path: List[Tuple[int, int]]           # visited (instances, batch) points, in order
    evaluated: int                        # distinct points measured


def search(measure: Callable[[int, int], Measurement], instance_counts: Sequence[int],
           batch_sizes: Sequence[int], sla_ms: float,
           power_w: float = float("inf")) -> SearchResult:
    """Gradient walk from (fewest instances, smallest batch).  Each step looks at
    larger batch / more instances / both, keeps those inside the latency and
    power bounds, and moves to the one that raises throughput most; it ends when
    none raises it.  Points are measured once."""
    cache: Dict[Tuple[int, int], Measurement] = {}

    def at(i: int, j: int) -> Measurement:
        if (i, j) not in cache:
            cache[(i, j)] = measure(instance_counts[i], batch_sizes[j])
        return cache[(i, j)]

    def in_bounds(x: Measurement) -> bool:
        return x.latency_ms < sla_ms and x.power_w < power_w

    i, j = 0, 0
    here = at(i, j)
    path = [(instance_counts[i], batch_sizes[j])]
    if not in_bounds(here):
        return SearchResult(None, None, None, path, len(cache))
    while True:
        step = None
        gain = 0.0
        for ni, nj in ((i, j + 1), (i + 1, j), (i + 1, j + 1)):
            if ni >= len(instance_counts) or nj >= len(batch_sizes):
                continue
            cand = at(ni, nj)
            if in_bounds(cand) and cand.qps - here.qps > gain:
                step, gain = (ni, nj), cand.qps - here.qps
        if step is None:
            return SearchResult(instance_counts[i], batch_sizes[j], here, path, len(cache))
        i, j = step
        here = at(i, j)
        path.append((instance_counts[i], batch_sizes[j]))


def measure_point(models, streams, batches_by_size, instances: int, batch: int,
                  rounds: int = 60, warmup: int = 8) -> Measurement:
    """One (instances, batch) point on the GPU.  models / streams: at least
    `instances` RecModel objects sharing tables and as many concurrent streams;
    batches_by_size[batch]: list of (dense, indices, lengths, logits) device tuples."""
    import numpy as np
    import torch
    data = batches_by_size[batch]

    def one_round(r: int) -> None:
        for k in range(instances):
            d, idx, lens, out = data[(r * instances + k) % len(data)]
            with torch.cuda.stream(streams[k]):
                models[k].forward(d, idx, lens, out[k])
        torch.cuda.synchronize()

    for r in range(warmup):
        one_round(r)
    lat = np.empty(rounds)
    for r in range(rounds):
        t = time.perf_counter()
        one_round(r)
        lat[r] = time.perf_counter() - t
    return Measurement(qps=instances * batch / float(lat.mean()),
                       latency_ms=float(np.percentile(lat, 99) * 1e3))
