"""Accelerator-side parallelism search: the oracle's Algorithm 1 against the
exhaustive definition on surfaces with the shape the paper reports (throughput
and tail latency convex over co-location and batch size), and the package's
scheduler against the oracle, step by step."""
import numpy as np
import pytest

from oracle import search_oracle as so
from paper_2203_07424_amd import scheduler


def surface(seed, n_m=4, n_d=8, peak=None):
    """Throughput rising then falling along both axes, latency growing with both."""
    g = np.random.default_rng(seed)
    pm = peak[0] if peak else g.integers(0, n_m)
    pd = peak[1] if peak else g.integers(0, n_d)
    a, b = g.uniform(0.5, 2.0, 2)
    m = np.arange(n_m)[:, None]
    d = np.arange(n_d)[None, :]
    qps = 1000.0 - a * 40.0 * (m - pm) ** 2 - b * 10.0 * (d - pd) ** 2
    lat = 0.5 + 0.8 * m + 0.15 * 2.0 ** d
    return qps, lat


def as_measure(qps, lat):
    return lambda mi, di: (float(qps[mi, di]), float(lat[mi, di]), 0.0)


@pytest.mark.parametrize("seed", range(12))
def test_algorithm1_reaches_the_exhaustive_optimum_on_convex_surfaces(seed):
    qps, lat = surface(seed)
    for L in (1e9, 20.0, 5.0, 1.2):
        got, path = so.algorithm1(as_measure(qps, lat), 4, 8, L)
        want, want_qps = so.exhaustive(as_measure(qps, lat), 4, 8, L)
        assert got is not None and want is not None
        assert path[0] == (0, 0) and path[-1] == got
        # every move raises throughput and stays within the bound
        for p, q in zip(path, path[1:]):
            assert qps[q] > qps[p] and lat[q] < L
            assert (q[0] - p[0], q[1] - p[1]) in ((0, 1), (1, 0), (1, 1))
        if L == 1e9:
            assert got == want                      # unconstrained: the peak itself
        else:
            assert lat[got] < L and qps[got] <= want_qps


def test_algorithm1_known_walk():
    qps = np.array([[10, 20, 30, 25], [15, 40, 35, 20], [12, 30, 50, 10]], float)
    lat = np.ones((3, 4))
    got, path = so.algorithm1(as_measure(qps, lat), 3, 4, 2.0)
    assert path == [(0, 0), (1, 1), (2, 2)] and got == (2, 2)
    lat[2, 2] = 5.0                                 # the peak breaks the SLA
    got, path = so.algorithm1(as_measure(qps, lat), 3, 4, 2.0)
    assert path == [(0, 0), (1, 1)] and got == (1, 1)     # (1,2) and (2,1) lose throughput
    lat[0, 0] = 9.0                                 # even the origin is out of bound
    assert so.algorithm1(as_measure(qps, lat), 3, 4, 2.0)[0] is None
    assert so.exhaustive(as_measure(qps, lat), 3, 4, 2.0) == ((1, 1), 40.0)


def test_power_bound_is_honoured():
    qps, lat = surface(3, peak=(3, 7))
    power = 100.0 + 50.0 * np.arange(4)[:, None] + 5.0 * np.arange(8)[None, :]
    meas = lambda mi, di: (float(qps[mi, di]), float(lat[mi, di]), float(power[mi, di]))
    got, path = so.algorithm1(meas, 4, 8, 1e9, P=180.0)
    assert all(power[p] < 180.0 for p in path) and got[0] <= 1


@pytest.mark.parametrize("seed", range(20))
def test_scheduler_follows_the_oracle_step_by_step(seed):
    g = np.random.default_rng(100 + seed)
    if seed % 2:
        qps, lat = surface(seed)
    else:                                            # arbitrary, non-convex tables too
        qps = g.uniform(0, 100, (4, 8))
        lat = g.uniform(0, 10, (4, 8))
    ms, ds = [1, 2, 3, 4], [64 << k for k in range(8)]
    L = float(g.choice([3.0, 6.0, 1e9]))
    calls = []

    def measure(m, d):
        calls.append((m, d))
        i, j = ms.index(m), ds.index(d)
        return scheduler.Measurement(float(qps[i, j]), float(lat[i, j]))
    res = scheduler.search(measure, ms, ds, L)
    got, path = so.algorithm1(as_measure(qps, lat), 4, 8, L)
    assert res.path == [(ms[i], ds[j]) for i, j in path]
    if got is None:
        assert res.instances is None and res.batch is None
    else:
        assert (res.instances, res.batch) == (ms[got[0]], ds[got[1]])
        assert res.measurement.qps == qps[got]
    assert len(calls) == len(set(calls)) == res.evaluated      # each point measured once
