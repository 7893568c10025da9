#!/usr/bin/env python3
"""Throughput of the DLRM-class forward pass on one MI355X.

One step = one rec_forward() over one synthetic batch: offsets scan, embedding
bag pooling, Bottom-FC, pairwise-dot interaction, Predict-FC.  Inputs and
tables are resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--steps K] [--warmup W] [--workload rmc2] [--uniform]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth

# HBM traffic of one pooling launch from rocprofv3 counter runs (FETCH_SIZE and
# WRITE_SIZE, each scaled by what it reads for a plain 1 GiB copy: 2.000 and
# 1.000), see profiles/pool_rmc2_counters.md.  Valid only for the kernel source
# the counters were taken with; reported as null once csrc/pool.hip differs.
POOL_TRAFFIC = {
    "sha256": "c49be4a068716d219cedf3b3a32fc300e91a6a0b40a9179c618037605bf46205",
    ("rmc2", 4096): {"fetch_bytes": 553996796.0, "write_bytes": 41943050.0},
    ("rmc2-uniform", 4096): {"fetch_bytes": 1707535117.0, "write_bytes": 41943198.0},
}


def measured_pool_traffic(w):
    import hashlib
    src = os.path.join(ROOT, "paper_2203_07424_amd", "csrc", "pool.hip")
    rec = POOL_TRAFFIC.get((w.name, w.batch))
    if rec is None or not os.path.exists(src):
        return None
    with open(src, "rb") as f:
        if hashlib.sha256(f.read()).hexdigest() != POOL_TRAFFIC["sha256"]:
            return None
    return rec["fetch_bytes"] + rec["write_bytes"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_pool_bytes(w, batch) -> int:
    """Bytes the pooling launch must move: gathered rows, their ids, the bag
    offsets, and the pooled vectors it writes."""
    elt = 2 if w.table_dtype == "f16" else 4
    bags = w.num_tables * w.batch
    return (batch.nnz * w.emb_dim * elt + batch.nnz * 4 + (bags + 1) * 4
            + bags * w.emb_dim * 4)


def cpu_baseline(w, batch, bottom, top, n_samples: int) -> dict:
    """The CPU oracle, as it stands, on a slice of the same batch."""
    import numpy as np
    from oracle import rec_oracle as orc
    from paper_2203_07424_amd import synth
    n_samples = min(n_samples, w.batch)
    sub = synth.slice_samples(w, batch, np.arange(n_samples))
    tabs, cidx = synth.compact_tables(w, sub, n_samples)
    cores = len(os.sched_getaffinity(0))
    threads = orc.set_threads(cores)
    t0 = time.perf_counter()
    orc.forward(sub.dense, tabs, cidx, sub.lengths, bottom, top)
    dt = time.perf_counter() - t0
    return {"value": n_samples / dt, "unit": "samples/s", "cores": threads, "kind": "oracle",
            "sample": f"first {n_samples} samples of batch 0 of {w.name} (rows they touch "
                      f"materialised in compact tables), whole forward, {dt:.2f} s wall"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="rmc2")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--uniform", action="store_true", help="uniform ids instead of Zipf")
    ap.add_argument("--batches", type=int, default=4, help="distinct input batches cycled")
    ap.add_argument("--cpu-samples", type=int, default=1024)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a kernel of known "
                         "traffic to scale hardware counters by)")
    ap.add_argument("--overlap", action="store_true",
                    help="run Bottom-FC on the library's side stream beside scan and pooling")
    ap.add_argument("--event-period", type=int, default=10,
                    help="bracket the stages of every N-th timed step with HIP events")
    ap.add_argument("--no-stage-events", action="store_true",
                    help="do not bracket stages with events inside the timed region")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1")
        return 2

    import numpy as np
    import torch
    from paper_2203_07424_amd import binding, synth

    w = synth.WORKLOADS[args.workload]
    if args.batch:
        w = w.with_batch(args.batch)
    if args.uniform:
        w = w.with_uniform_indices()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    t0 = time.time()
    hi = w.pooling[1] if w.pooling[0] == "fixed" else w.pooling[3]
    m = binding.RecModel(w.num_tables, w.emb_dim, [w.rows] * w.num_tables, w.table_dtype,
                         w.num_dense, list(w.bottom), list(w.top), w.batch,
                         w.batch * w.num_tables * hi)
    tdt = torch.float16 if w.table_dtype == "f16" else torch.float32
    for t in range(w.num_tables):
        tab = torch.empty((w.rows, w.emb_dim), dtype=tdt, device=dev)
        assert binding.rec_synth_fill_table(tab, w.seed, t) == binding.REC_OK
        m.load_table(t, tab)
    bottom, top = synth.draw_mlp(w, "bottom"), synth.draw_mlp(w, "top")
    for i, (W, b) in enumerate(bottom):
        m.load_mlp(binding.REC_BOTTOM, i, torch.from_numpy(W), torch.from_numpy(b))
    for i, (W, b) in enumerate(top):
        m.load_mlp(binding.REC_TOP, i, torch.from_numpy(W), torch.from_numpy(b))
    if args.overlap:
        m.set_option(binding.REC_OPT_OVERLAP_DENSE, 1)
    torch.cuda.synchronize()
    log(f"model {w.name}: {w.num_tables} x {w.rows} x {w.emb_dim} {w.table_dtype} resident "
        f"({time.time() - t0:.1f} s)")

    cdf = synth.zipf_cdf(w.rows, float(w.index_dist[1])) if w.index_dist[0] == "zipf" else None
    host_batches = [synth.draw_batch(w, i, cdf) for i in range(args.batches)]
    dev_batches = [(torch.from_numpy(b.dense).to(dev), torch.from_numpy(b.indices).to(dev),
                    torch.from_numpy(b.lengths).to(dev)) for b in host_batches]
    logits = torch.empty(w.batch, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    log(f"{args.batches} batches of {w.batch} resident, nnz[0] = {host_batches[0].nnz} "
        f"({time.time() - t0:.1f} s)")

    def step(i):
        d, idx, lens = dev_batches[i % len(dev_batches)]
        m.forward(d, idx, lens, logits)

    if args.calibration_copy_mib:
        n = args.calibration_copy_mib << 20
        src = torch.full((n,), 1, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    st, pos = m.check()
    assert st == binding.REC_OK, (st, pos)

    use_events = not args.no_stage_events
    n_timed = (args.steps + args.event_period - 1) // args.event_period
    if use_events:
        m.set_profiling(n_timed, args.event_period)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start

    ms_per_step = elapsed * 1e3 / args.steps
    value = w.batch * args.steps / elapsed

    stage_avg = None
    roofline = None
    if use_events:
        acc = np.zeros(binding.REC_NUM_STAGES)
        for j in range(n_timed):
            acc += np.array(list(m.stage_ms(j).values()))
        stage_avg = dict(zip(binding.STAGE_NAMES, (acc / n_timed).tolist()))
        m.set_profiling(0)
        pool_bytes = np.mean([algorithmic_pool_bytes(w, host_batches[i % len(host_batches)])
                              for i in range(0, args.steps, args.event_period)])
        achieved = pool_bytes / (stage_avg["pool"] * 1e-3) / 1e9
        roofline = {"kernel": "pool_kernel (embedding-bag gather-reduce)", "bound": "hbm",
                    "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_pool_traffic(w),
                    "bytes_per_launch": float(pool_bytes), "avg_launch_ms": stage_avg["pool"],
                    "launches_timed": n_timed}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, host_batches[0], bottom, top, args.cpu_samples)

    out = {
        "metric": "samples/sec per GPU + embedding-bag HBM GB/s (% of peak), RMC2-style",
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 tables -> f32 accumulate; bf16 MFMA -> f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.num_tables} tables x {w.rows} rows x dim {w.emb_dim} "
                               f"{w.table_dtype}, pooling {w.pooling}, ids {w.index_dist}, "
                               f"bottom {list(w.bottom)}, top {list(w.top)}",
                   "batch": w.batch, "distinct_batches": args.batches,
                   "mean_nnz": float(np.mean([b.nnz for b in host_batches]))},
        "roofline": roofline, "cpu_baseline": cpu, "stage_ms": stage_avg,
    }
    print(json.dumps(out), flush=True)
    m.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
