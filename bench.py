#!/usr/bin/env python3
"""Throughput of the DLRM-class forward pass on one MI355X.

One step = one rec_forward() over one synthetic batch: offsets scan, embedding
bag pooling, Bottom-FC, pairwise-dot interaction, Predict-FC.  Inputs and
tables are resident in HBM before the timed region.  Prints ONE JSON line.

Default run (workload rmc2, the configuration the metric is quoted on):
  value               K steps through the pipelined model (four streams: scan and
                      Bottom-FC, two pooling streams taken in turn, interaction and
                      Predict-FC; four batches in flight), drained and synchronised
  in_order            the same K steps with everything in order on one stream
  sustained           the pipelined loop kept up for at least two seconds
  latency_ms          one batch at a time, host launch and synchronisation included
  stage_ms, mlp_mfma  HIP-event brackets around every stage of in-order forwards
  roofline            the pooling kernel on the uniform-id twin (no reuse for the
                      caches to serve): algorithmic bytes / launch time against the
                      HBM peak
  roofline_zipf       the same kernel on the headline's skewed ids, where the caches
                      serve most rows: algorithmic rate, and the bytes that must come
                      from HBM at least (unique rows + ids) against the peak
  co_located          two in-order instances sharing the tables, a stream each
  other_workloads     short legs of tiny, rmc1, rmc3, mtwnd and the batch-size sweep
                      of rmc2-large (154 GB resident) with its latency-bounded rate
  cpu_baseline        the CPU oracle, as it stands, on a bounded sample

  python bench.py [--steps K] [--warmup W] [--workload rmc2] [--uniform]
  python bench.py --workload rmc2-large --latency-sweep
  python bench.py --search
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate

# HBM traffic of one pooling launch from rocprofv3 counter runs (FETCH_SIZE and
# WRITE_SIZE, each scaled by what it reads for a plain 1 GiB copy: 2.000 and
# 1.000), see profiles/pool_rmc2_counters.md; Zipf ids with cached row loads,
# the uniform twin with non-temporal ones.  These are figures from a profile, not
# of this run, and hold only for the kernel source the counters were taken with:
# reported as null once csrc/pool.hip differs.
POOL_TRAFFIC = {
    "sha256": "ab1846d96d7f5f0750d6a6ca9f670f1d5e0548b462a4c702c976c977754e84da",
    ("rmc2", 4096): {"fetch_bytes": 553867622.0, "write_bytes": 41943056.0},
    ("rmc2-uniform", 4096): {"fetch_bytes": 1721570714.0, "write_bytes": 41943100.0},
}


def profiled_pool_traffic(w, streaming):
    import hashlib
    if streaming != (w.index_dist[0] == "uniform"):   # the counters were taken with the automatic choice
        return None
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


def dtype_string(w) -> str:
    tab = "f16" if w.table_dtype == "f16" else "f32"
    s = f"{tab} tables -> f32 pooling sums; bf16 MFMA -> f32 accumulate (FC layers)"
    if w.interaction == "dot":
        s += "; interaction: f32 operands split into two bf16 planes on bf16 MFMA (16 significant bits) -> bf16"
    return s


def workload_string(w) -> str:
    return (f"{w.name}: {w.num_tables} tables x {w.rows} rows x dim {w.emb_dim} {w.table_dtype}, "
            f"pooling {w.pooling}, ids {w.index_dist}, bottom {list(w.bottom)}, top {list(w.top)}"
            + (f" x {w.towers} towers, concatenation" if w.interaction == "concat" else ""))


def algorithmic_pool_bytes(w, batch) -> int:
    """Bytes the pooling launch must move: gathered rows, their ids, the bag
    offsets, and the pooled vectors it writes (counted: yes)."""
    elt = 2 if w.table_dtype == "f16" else 4
    bags = w.num_tables * w.batch
    out_elt = 2 if w.interaction == "concat" else 4
    return (batch.nnz * w.emb_dim * elt + batch.nnz * 4 + (bags + 1) * 4
            + bags * w.emb_dim * out_elt)


def compulsory_pool_bytes(w, batch) -> int:
    """Bytes that must come from or go to HBM at least: every distinct row once,
    the ids, the offsets and the pooled vectors."""
    import numpy as np
    elt = 2 if w.table_dtype == "f16" else 4
    bags = w.num_tables * w.batch
    per_table = batch.lengths.reshape(w.num_tables, w.batch).sum(axis=1, dtype=np.int64)
    pos, uniq = 0, 0
    for t in range(w.num_tables):
        n = int(per_table[t])
        uniq += np.unique(batch.indices[pos:pos + n]).size
        pos += n
    out_elt = 2 if w.interaction == "concat" else 4
    return uniq * w.emb_dim * elt + batch.nnz * 4 + (bags + 1) * 4 + bags * w.emb_dim * out_elt


def repeats_within_chunks(w, batch) -> dict:
    """How many lookups repeat an id that the same wave already holds: the pooling
    kernel takes a bag 64 ids at a time, 8 rows per wave-wide load.  What loading
    each distinct id of a chunk once (and scaling by its count) could save, before
    the cost of finding the repeats."""
    import numpy as np
    lengths = batch.lengths.astype(np.int64)
    bag_of = np.repeat(np.arange(lengths.size, dtype=np.int64), lengths)
    starts = np.concatenate(([0], np.cumsum(lengths)[:-1]))
    pos = np.arange(batch.nnz, dtype=np.int64) - starts[bag_of]
    chunk = bag_of * 4 + pos // 64                      # bags hold at most 200 ids: 4 chunks
    key = np.sort(chunk << 32 | batch.indices[:batch.nnz].astype(np.int64))
    first = np.ones(key.size, dtype=bool)
    first[1:] = key[1:] != key[:-1]
    n_chunks = int(chunk.max()) + 1
    total = np.bincount(chunk, minlength=n_chunks)
    distinct = np.bincount(key[first] >> 32, minlength=n_chunks)
    loads, loads_distinct = ((total + 7) // 8).sum(), ((distinct + 7) // 8).sum()
    return {"lookups_repeating_an_id_of_their_chunk": float(1.0 - distinct.sum() / total.sum()),
            "wave_wide_row_loads_saved": float(1.0 - loads_distinct / loads),
            "what": "batch 0; chunk = the 64 ids of a bag a wave holds at a time, 8 rows per wave-wide load"}


def cpu_baseline(w, batches, bottom, top, n_samples: int) -> dict:
    """The CPU oracle, as it stands, on the first n_samples samples of each of
    the given batches (a bounded sample: tens of core-seconds of CPU work)."""
    import numpy as np
    from oracle import rec_oracle as orc
    from paper_2203_07424_amd import synth
    n_samples = min(n_samples, w.batch)
    cores = len(os.sched_getaffinity(0))
    threads = orc.set_threads(cores)
    dt = 0.0
    for batch in batches:
        sub = synth.slice_samples(w, batch, np.arange(n_samples)) if n_samples < w.batch else batch
        tabs, cidx = synth.compact_tables(w, sub, n_samples)
        t0 = time.perf_counter()
        if w.interaction == "concat":
            orc.forward_towers(sub.dense, tabs, cidx, sub.lengths, bottom, top)
        else:
            orc.forward(sub.dense, tabs, cidx, sub.lengths, bottom, top)
        dt += time.perf_counter() - t0
    total = n_samples * len(batches)
    # one thread, on a smaller slice, for the per-core rate
    n1 = min(256, n_samples)
    sub = synth.slice_samples(w, batches[0], np.arange(n1))
    tabs, cidx = synth.compact_tables(w, sub, n1)
    orc.set_threads(1)
    t0 = time.perf_counter()
    if w.interaction == "concat":
        orc.forward_towers(sub.dense, tabs, cidx, sub.lengths, bottom, top)
    else:
        orc.forward(sub.dense, tabs, cidx, sub.lengths, bottom, top)
    dt1 = time.perf_counter() - t0
    orc.set_threads(threads)
    return {"value": total / dt, "unit": "samples/s", "cores": threads, "kind": "oracle",
            "single_thread": {"value": n1 / dt1, "unit": "samples/s", "sample": f"first {n1} samples of batch 0, {dt1:.2f} s"},
            "sample": f"first {n_samples} samples of each of {len(batches)} batches of {w.name} (rows they "
                      f"touch materialised in compact tables, which is not timed), whole forward, "
                      f"{dt:.2f} s wall on {threads} threads"}


FUSE_MLP = "auto"   # --fuse-mlp: how runs of narrow FC layers are launched


def build_model(binding, synth, torch, w, max_batch, share_tables=None, pipeline=False, dense_stream=None,
                pool_streams=(None, None)):
    """Model of workload `w` with tables filled on the device (or shared with
    the model `share_tables`) and packed MLPs."""
    dev = torch.device("cuda:0")
    hi = w.pooling[1] if w.pooling[0] == "fixed" else w.pooling[3]
    m = binding.RecModel(w.num_tables, w.emb_dim, [w.rows] * w.num_tables, w.table_dtype,
                         w.num_dense, list(w.bottom), list(w.top), max_batch,
                         min(max_batch * w.num_tables * hi, 2 ** 31 - 1),
                         interaction=w.interaction, towers=w.towers, pipeline=pipeline,
                         dense_stream=dense_stream, pool_streams=pool_streams)
    tdt = torch.float16 if w.table_dtype == "f16" else torch.float32
    for t in range(w.num_tables):
        if share_tables is not None:
            tab = share_tables.tables[t]
        else:
            tab = torch.empty((w.rows, w.emb_dim), dtype=tdt, device=dev)
            assert binding.rec_synth_fill_table(tab, w.seed, t) == binding.REC_OK
        m.load_table(t, tab)
    bottom = synth.draw_mlp(w, "bottom")
    towers = [synth.draw_mlp(w, "top", k) for k in range(w.towers)]
    for i, (W, b) in enumerate(bottom):
        m.load_mlp(binding.REC_BOTTOM, i, torch.from_numpy(W), torch.from_numpy(b))
    for k, tower in enumerate(towers):
        for i, (W, b) in enumerate(tower):
            m.load_mlp(binding.REC_TOP + k, i, torch.from_numpy(W), torch.from_numpy(b))
    if FUSE_MLP != "auto":
        m.set_option(binding.REC_OPT_FUSE_MLP, 2 if FUSE_MLP == "on" else 0)
    torch.cuda.synchronize()
    # the oracle's pairwise-dot forward takes one stack, its tower forward a list of them
    return m, bottom, (towers if w.interaction == "concat" else towers[0])


def new_logits(torch, w, batch, dev):
    shape = (batch,) if w.towers == 1 else (batch, w.towers)
    return torch.empty(shape, dtype=torch.float32, device=dev)


def pick_concurrent_streams(torch, dev, n):
    """n streams that really run side by side.

    HIP deals its few hardware queues to streams in creation order, so two
    streams may share one and then serialise.  Each candidate is probed with a
    pair of spin kernels: on separate queues the pair takes about as long as
    one of them."""
    cand = [torch.cuda.Stream(device=dev) for _ in range(8)]
    if n <= 1:
        return cand[:1]
    spin = 2_000_000

    def pair_ms(a, b):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for s in (a, b):
            with torch.cuda.stream(s):
                torch.cuda._sleep(spin)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3

    pair_ms(cand[0], cand[1])                      # warm-up
    alone = min(pair_ms(cand[0], cand[0]) for _ in range(2)) / 2
    chosen = [cand[0]]
    for c in cand[1:]:
        if len(chosen) == n:
            break
        if all(min(pair_ms(c, o) for _ in range(2)) < 1.5 * alone for o in chosen):
            chosen.append(c)
    if len(chosen) < n:
        log(f"only {len(chosen)} concurrent streams found for {n} instances")
        chosen += [cand[i] for i in range(8) if cand[i] not in chosen][:n - len(chosen)]
    return chosen


def make_batches(torch, synth, wl, n, first_id, dev, workers=8):
    """n distinct batches of workload wl: host copies and device-resident tensors."""
    from concurrent.futures import ThreadPoolExecutor
    cdf = synth.zipf_cdf(wl.rows, float(wl.index_dist[1])) if wl.index_dist[0] == "zipf" else None
    if n >= workers:
        with ThreadPoolExecutor(workers) as ex:
            hb = list(ex.map(lambda i: synth.draw_batch(wl, first_id + i, cdf), range(n)))
    else:
        hb = [synth.draw_batch(wl, first_id + i, cdf, workers=workers) for i in range(n)]
    db = [(torch.from_numpy(b.dense).to(dev), torch.from_numpy(b.indices).to(dev),
           torch.from_numpy(b.lengths).to(dev)) for b in hb]
    torch.cuda.synchronize()
    return hb, db


def run_steps(torch, model, stream, db, outs, steps, first=0):
    """steps forwards of `model` on `stream` over the batches in turn, drained
    and synchronised; returns seconds."""
    torch.cuda.synchronize()
    t = time.perf_counter()
    with torch.cuda.stream(stream):
        for i in range(first, first + steps):
            model.forward(*db[i % len(db)], outs[i % len(outs)])
        model.drain()
    torch.cuda.synchronize()
    return time.perf_counter() - t


def stage_profile(torch, binding, np, model, stream, db, n):
    """n in-order forwards, every stage bracketed with HIP events on `stream`.
    Returns (mean ms per stage, per-forward pool ms, index of the batch each used)."""
    with torch.cuda.stream(stream):
        for i in range(5):
            model.forward(*db[i % len(db)])
        model.drain()
        torch.cuda.synchronize()
        model.set_profiling(n, 1)
        outs = [None] * len(db)
        for i in range(n):
            outs[i % len(db)] = model.forward(*db[i % len(db)], outs[i % len(db)])
        model.drain()
    torch.cuda.synchronize()
    rows = np.array([list(model.stage_ms(j).values()) for j in range(n)])
    model.set_profiling(0)
    mean = dict(zip(binding.STAGE_NAMES, rows.mean(axis=0).tolist()))
    return mean, rows[:, binding.STAGE_NAMES.index("pool")], [i % len(db) for i in range(n)]


def latency_profile(torch, np, model, stream, db, out, iters, warmup=10):
    """One batch in flight at a time: per-batch latency, host launch and synchronisation included."""
    with torch.cuda.stream(stream):
        for i in range(warmup):
            model.forward(*db[i % len(db)], out)
        model.drain()
        torch.cuda.synchronize()
        lat = np.empty(iters)
        for i in range(iters):
            t = time.perf_counter()
            model.forward(*db[i % len(db)], out)
            model.drain()
            stream.synchronize()
            lat[i] = time.perf_counter() - t
    return {"p50": float(np.percentile(lat, 50) * 1e3), "p99": float(np.percentile(lat, 99) * 1e3),
            "min": float(lat.min() * 1e3), "max": float(lat.max() * 1e3), "mean": float(lat.mean() * 1e3),
            "iterations": iters}


SUSTAINED_RANDOM_TFLOPS = None   # set by main() once mfma_sustained() has run


def mlp_mfma(wl, avg):
    """Matrix-unit use of the FC stages: unpadded 2*M*N*K of the stage's layers over
    its HIP-event interval (which includes one event record and, for small
    layers, mostly launch latency) against the bf16 MFMA peak.  bottom_first and
    top_first bracket a single launch each."""
    def flops(widths):
        return sum(2.0 * wl.batch * widths[i] * widths[i + 1] for i in range(len(widths) - 1))
    out = {}
    for stage, widths, mult in (("bottom_first", wl.bottom[:2], 1), ("bottom_rest", wl.bottom[1:], 1),
                                ("top_first", wl.top[:2], wl.towers), ("top_rest", wl.top[1:], wl.towers)):
        f = flops(widths) * mult
        if f > 0 and avg.get(stage, 0) > 0:
            tf = f / (avg[stage] * 1e-3) / 1e12
            out[stage] = {"gflop": f / 1e9, "ms": avg[stage], "tflops": tf,
                          "frac_of_bf16_peak": tf / MFMA_BF16_PEAK_TFLOPS}
            if SUSTAINED_RANDOM_TFLOPS:
                out[stage]["frac_of_sustained_rate_on_random_operands"] = tf / SUSTAINED_RANDOM_TFLOPS
    return out


def library_gemm_yardstick(torch, M, N, K, dev, reps=30):
    """What the vendor's GEMM library (through torch.matmul) reaches on bf16
    operands of one layer's shape on this machine: a yardstick beside the published
    peak, like the device copy is for HBM.  Not part of the forward pass."""
    a = torch.randn(M, K, device=dev, dtype=torch.bfloat16)
    b = torch.randn(N, K, device=dev, dtype=torch.bfloat16)
    for _ in range(5):
        c = a @ b.t()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        c = a @ b.t()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
    del a, b, c
    return {"shape_m_n_k": [M, N, K], "ms": ms, "tflops": tf, "frac_of_bf16_peak": tf / MFMA_BF16_PEAK_TFLOPS,
            "what": "torch.matmul (vendor GEMM library) on bf16 operands of the same shape, back to back, by events; "
                    "no bias, no activation"}


def mfma_sustained(torch, binding, dev):
    """The bf16 matrix rate this device sustains on nothing but matrix
    instructions (rec_probe_mfma: register operands, 8 wavefronts per compute
    unit): on constant operands, on random ones, and on random ones with a quarter
    of the compute units busy.  With the whole chip busy the rate is power-limited
    and depends on the operand bits, so the middle figure, not the published peak,
    is what a GEMM on real data can reach here."""
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    out = {"compute_units": cus}
    iters = 2000
    for label, rnd, blocks in (("constant_operands", False, cus), ("random_operands", True, cus),
                               ("random_operands_quarter_of_the_chip", True, max(1, cus // 4))):
        assert binding.rec_probe_mfma(rnd, blocks, 200, sink) == binding.REC_OK     # warm-up
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        assert binding.rec_probe_mfma(rnd, blocks, iters, sink) == binding.REC_OK
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        flops = float(blocks) * 8 * iters * 32 * 32768
        tf = flops / (ms * 1e-3) / 1e12
        out[label] = {"blocks": blocks, "ms": ms, "tflops": tf,
                      "tflops_per_compute_unit": tf / blocks,
                      "frac_of_bf16_peak": tf / (MFMA_BF16_PEAK_TFLOPS * blocks / cus)}
    out["what"] = ("rec_probe_mfma: v_mfma_f32_32x32x16_bf16 on register operands only, one workgroup of 8 wavefronts "
                   "per compute unit; fractions are of the published peak scaled to the compute units in use")
    return out


def widest_layer_yardstick(torch, wl, dev):
    """The library yardstick for the widest matrix product of the workload (first
    Bottom-FC layer, or first Predict-FC layer of all towers side by side)."""
    cands = []
    if len(wl.bottom) > 1:
        cands.append(("bottom_first", wl.batch, wl.bottom[1], wl.bottom[0]))
    cands.append(("top_first", wl.batch, wl.top[1] * wl.towers, wl.top[0]))
    stage, M, N, K = max(cands, key=lambda c: c[1] * c[2] * c[3])
    if 2.0 * M * N * K < 1e10:      # small layers are launch-bound either way
        return None
    y = library_gemm_yardstick(torch, M, N, K, dev)
    y["stage"] = stage
    return y


def pool_roofline(np, wl, hb, used, pool_ms, streaming, kind="algorithmic"):
    """The pooling kernel against the HBM peak: bytes per launch over the mean
    launch time of the timed launches."""
    fn = algorithmic_pool_bytes if kind == "algorithmic" else compulsory_pool_bytes
    per_batch = [fn(wl, b) for b in hb]
    nbytes = float(np.mean([per_batch[i] for i in used]))
    ms = float(np.mean(pool_ms))
    gbps = nbytes / (ms * 1e-3) / 1e9
    return {"kernel": "pool_kernel (embedding-bag gather-reduce)", "bound": "hbm", "achieved": gbps,
            "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
            "traffic": profiled_pool_traffic(wl, streaming), "bytes_per_launch": nbytes,
            "bytes_counted": "gathered rows + ids + offsets + pooled vectors written" if kind == "algorithmic"
                             else "distinct rows + ids + offsets + pooled vectors written",
            "avg_launch_ms": ms, "min_launch_ms": float(np.min(pool_ms)), "launches_timed": int(len(pool_ms)),
            "distinct_batches": len(hb), "workload": wl.name,
            "row_loads": "non-temporal" if streaming else "cached"}


def short_leg(torch, binding, synth, np, name, args, dev, streams):
    """One of the other workloads: throughput in order and pipelined, per-batch
    latency, stage times, matrix-unit use of its FC stages, pooling rate."""
    w = synth.WORKLOADS[name]
    t0 = time.time()
    m, _, _ = build_model(binding, synth, torch, w, w.batch)
    pm, _, _ = build_model(binding, synth, torch, w, w.batch, share_tables=m, pipeline=True,
                           dense_stream=streams[3], pool_streams=(streams[1], streams[2]))
    streaming = w.index_dist[0] == "uniform"
    for mm in (m, pm):
        mm.set_option(binding.REC_OPT_STREAM_ROWS, int(streaming))
    hb, db = make_batches(torch, synth, w, 8, 0, dev)
    outs = [new_logits(torch, w, w.batch, dev) for _ in range(4)]
    steps = args.other_steps
    res = {"workload": workload_string(w), "batch": w.batch, "dtype": dtype_string(w), "steps": steps,
           "distinct_batches": len(hb)}
    for label, model in (("in_order", m), ("pipelined", pm)):
        run_steps(torch, model, streams[0], db, outs, 20)
        dt = run_steps(torch, model, streams[0], db, outs, steps)
        res[label] = {"value": w.batch * steps / dt, "unit": "samples/s", "ms_per_step": dt * 1e3 / steps}
        assert model.check() == (binding.REC_OK, -1)
    res["value"] = max(res["in_order"]["value"], res["pipelined"]["value"])
    res["latency_ms"] = latency_profile(torch, np, m, streams[0], db, outs[0], 100)
    avg, pool_ms, used = stage_profile(torch, binding, np, m, streams[0], db, 32)
    res["stage_ms"] = avg
    res["mlp_mfma"] = mlp_mfma(w, avg)
    y = widest_layer_yardstick(torch, w, dev)
    if y:
        res["library_gemm_yardstick"] = y
    res["pooling"] = pool_roofline(np, w, hb, used, pool_ms, streaming)
    if w.index_dist[0] == "zipf":      # cache-served: an algorithmic rate, not a fraction of the HBM peak
        res["pooling"]["algorithmic_gbps"] = res["pooling"].pop("achieved")
        for k in ("frac", "bound"):
            res["pooling"].pop(k)
    m.close()
    pm.close()
    log(f"  {name}: {res['value'] / 1e6:.2f} M samples/s ({time.time() - t0:.1f} s)")
    return res


PIPELINE_WINDOW = 4   # batches in flight in the pipelined closed loop: one per workspace frame


def windowed_pipeline_profile(torch, np, pm, streams, db, outs, n, warmup):
    """Closed loop through the pipelined model with PIPELINE_WINDOW batches in
    flight: batch i is enqueued once batch i - PIPELINE_WINDOW has finished.  A
    batch's latency runs from the moment the caller's stream reaches its call to
    the end of its last stage (an event on the dense stream)."""
    total = n + warmup
    begin = [torch.cuda.Event(enable_timing=True) for _ in range(total)]
    end = [torch.cuda.Event(enable_timing=True) for _ in range(total)]
    t = 0.0
    torch.cuda.synchronize()
    with torch.cuda.stream(streams[0]):
        for i in range(total):
            if i >= PIPELINE_WINDOW:
                end[i - PIPELINE_WINDOW].synchronize()
            if i == warmup:
                t = time.perf_counter()
            begin[i].record(streams[0])
            pm.forward(*db[i % len(db)], outs[i % len(outs)])
            end[i].record(pm.dense_stream)
        pm.drain()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t
    lat = np.array([begin[i].elapsed_time(end[i]) for i in range(warmup, total)])
    return {"p50": float(np.percentile(lat, 50)), "p99": float(np.percentile(lat, 99)), "max": float(lat.max()),
            "mean": float(lat.mean()), "seconds": dt, "iterations": n}


def sweep_leg(torch, binding, synth, np, w0, sizes, iters, sla_ms, dev, streams, warmup=10):
    """Batch-size sweep: per-batch latency with one batch in flight and, through
    the pipelined model, with PIPELINE_WINDOW in flight (closed loops: queuing delay
    excluded), and the latency-bounded throughput (Sec. II-B) under sla_ms."""
    t0 = time.time()
    m, _, _ = build_model(binding, synth, torch, w0, max(sizes))
    pm, _, _ = build_model(binding, synth, torch, w0, max(sizes), share_tables=m, pipeline=True,
                           dense_stream=streams[3], pool_streams=(streams[1], streams[2]))
    log(f"  {w0.name} resident ({time.time() - t0:.1f} s)")
    rows = []
    for B in sizes:
        w = w0.with_batch(B)
        hb, db = make_batches(torch, synth, w, 2, 1000, dev)
        outs = [new_logits(torch, w, B, dev) for _ in range(PIPELINE_WINDOW)]
        lat = latency_profile(torch, np, m, streams[0], db, outs[0], iters, warmup)
        pl = windowed_pipeline_profile(torch, np, pm, streams, db, outs, iters, warmup)
        assert m.check() == (binding.REC_OK, -1) and pm.check() == (binding.REC_OK, -1)
        rows.append({"batch": B, "mean_nnz": float(np.mean([b.nnz for b in hb])), "p50_ms": lat["p50"],
                     "p99_ms": lat["p99"], "max_ms": lat["max"], "samples_per_s": B / (lat["mean"] * 1e-3),
                     "pipelined": {"in_flight": PIPELINE_WINDOW, "p50_ms": pl["p50"], "p99_ms": pl["p99"],
                                   "max_ms": pl["max"], "samples_per_s": B * iters / pl["seconds"]}})
        log(f"  B={B}: p50 {lat['p50']:.3f} ms p99 {lat['p99']:.3f} ms "
            f"{rows[-1]['samples_per_s'] / 1e6:.2f} M samples/s; pipelined p99 {pl['p99']:.3f} ms "
            f"{rows[-1]['pipelined']['samples_per_s'] / 1e6:.2f} M samples/s ({time.time() - t0:.1f} s)")
        del db, outs
    pm.close()
    m.close()

    def bounded(limit):
        cand = [(r["samples_per_s"], r["batch"], "one batch in flight") for r in rows if r["p99_ms"] <= limit]
        cand += [(r["pipelined"]["samples_per_s"], r["batch"], f"pipelined, {PIPELINE_WINDOW} batches in flight")
                 for r in rows if r["pipelined"]["p99_ms"] <= limit]
        return max(cand) if cand else None
    best, best50 = bounded(sla_ms), bounded(50.0)
    return {"workload": workload_string(w0), "dtype": dtype_string(w0), "sla_ms": sla_ms,
            "latency_bounded_samples_per_s": best[0] if best else None,
            "best_batch": best[1] if best else None, "best_mode": best[2] if best else None,
            "at_the_paper_s_50_ms_bound": {"samples_per_s": best50[0] if best50 else None,
                                           "best_batch": best50[1] if best50 else None,
                                           "best_mode": best50[2] if best50 else None},
            "iterations_per_batch_size": iters,
            "note": "closed loops: one batch in flight (latency includes the host's launch calls), and the "
                    f"pipelined model with {PIPELINE_WINDOW} batches in flight (latency from the caller's stream "
                    "reaching the call to the end of the batch's last stage); queuing delay excluded; p99 over "
                    "the timed iterations",
            "sweep": rows}


def latency_sweep(args) -> int:
    """--latency-sweep: the sweep alone, as the JSON line's subject."""
    import numpy as np
    import torch
    from paper_2203_07424_amd import binding, synth

    w0 = synth.WORKLOADS[args.workload]
    sizes = [int(x) for x in args.sweep_batches.split(",")]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    r = sweep_leg(torch, binding, synth, np, w0, sizes, args.sweep_iters, args.sla_ms, dev,
                  pick_concurrent_streams(torch, dev, 4), args.warmup)
    best = next((x for x in r["sweep"] if x["batch"] == r["best_batch"]), None)
    if best and r["best_mode"] != "one batch in flight":
        best = best["pipelined"]
    out = {"metric": f"latency-bounded samples/s per GPU at p99 <= {args.sla_ms} ms per batch",
           "value": r["latency_bounded_samples_per_s"], "unit": "samples/s", "n_gpus": 1,
           "steps": args.sweep_iters, "warmup": args.warmup,
           "ms_per_step": best["p50_ms"] if best else None, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": dtype_string(w0), "data": "synthetic",
           "config": {"workload": r["workload"], "best_batch": r["best_batch"], "mode": r["best_mode"],
                      "sla_ms": args.sla_ms, "note": r["note"]},
           "at_the_paper_s_50_ms_bound": r["at_the_paper_s_50_ms_bound"], "sweep": r["sweep"]}
    print(json.dumps(out), flush=True)
    return 0


def search_mode(args) -> int:
    """Gradient-based search (Algorithm 1, accelerator-side P_sp(M+D)) for the
    batch size and the number of co-located instances with the highest
    throughput under the SLA; optionally the full grid beside it."""
    import torch
    from paper_2203_07424_amd import binding, scheduler, synth

    w0 = synth.WORKLOADS[args.workload]
    sizes = [int(x) for x in args.sweep_batches.split(",")]
    counts = list(range(1, args.search_instances + 1))
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    t0 = time.time()
    m0, _, _ = build_model(binding, synth, torch, w0, max(sizes))
    models = [m0] + [build_model(binding, synth, torch, w0, max(sizes), share_tables=m0)[0]
                     for _ in counts[1:]]
    streams = pick_concurrent_streams(torch, dev, len(counts))
    data = {}
    for B in sizes:
        w = w0.with_batch(B)
        outs = [new_logits(torch, w, B, dev) for _ in counts]
        _, db = make_batches(torch, synth, w, 2, 2000, dev)
        data[B] = [(d, i, l, outs) for d, i, l in db]
    log(f"{len(counts)} instances of {w0.name}, batches {sizes} resident ({time.time() - t0:.1f} s)")
    memo = {}

    def measure(m, d):
        if (m, d) not in memo:
            memo[(m, d)] = scheduler.measure_point(models, streams, data, m, d, rounds=args.sweep_iters)
            x = memo[(m, d)]
            log(f"  instances {m} batch {d}: {x.qps / 1e6:.2f} M samples/s, p99 {x.latency_ms:.3f} ms")
        return memo[(m, d)]
    res = scheduler.search(measure, counts, sizes, args.sla_ms)
    grid = None
    if args.search_exhaustive:
        grid = [{"instances": m, "batch": d, "samples_per_s": measure(m, d).qps,
                 "p99_ms": measure(m, d).latency_ms} for m in counts for d in sizes]
    out = {"metric": f"latency-bounded samples/s per GPU at p99 <= {args.sla_ms} ms, gradient search over "
                     "(co-located instances, batch size)",
           "value": res.measurement.qps if res.measurement else None, "unit": "samples/s", "n_gpus": 1,
           "steps": args.sweep_iters, "warmup": 8,
           "ms_per_step": res.measurement.latency_ms if res.measurement else None,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": dtype_string(w0), "data": "synthetic",
           "config": {"workload": w0.name, "instances": res.instances, "batch": res.batch,
                      "sla_ms": args.sla_ms, "points_measured_by_search": res.evaluated,
                      "grid_points": len(counts) * len(sizes)},
           "path": res.path, "grid": grid}
    print(json.dumps(out), flush=True)
    for mm in models:
        mm.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="rmc2")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--uniform", action="store_true", help="uniform ids instead of Zipf")
    ap.add_argument("--batches", type=int, default=8, help="distinct input batches cycled")
    ap.add_argument("--mode", choices=["pipelined", "in-order"], default="pipelined",
                    help="what the timed region runs: the sparse-dense pipeline over four streams, "
                         "or everything in order on one stream")
    ap.add_argument("--colocated-leg", type=int, default=2,
                    help="instances of the co-located leg (0 or 1 = none)")
    ap.add_argument("--timed-launches", type=int, default=40,
                    help="forwards whose stages are bracketed with HIP events, per leg")
    ap.add_argument("--latency-iters", type=int, default=200)
    ap.add_argument("--sustain-seconds", type=float, default=2.0)
    ap.add_argument("--other-steps", type=int, default=200, help="steps of each other workload's leg")
    ap.add_argument("--no-other-workloads", action="store_true")
    ap.add_argument("--cpu-samples", type=int, default=4096)
    ap.add_argument("--cpu-batches", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a kernel of known "
                         "traffic to scale hardware counters by)")
    ap.add_argument("--hot-rows", type=int, default=0,
                    help="register the N most frequent rows of each table (profiled on two "
                         "batches that are not timed) so that pooling serves them from LDS")
    ap.add_argument("--graph", action="store_true",
                    help="record the distinct batches' forwards (in the chosen --mode) into one HIP graph "
                         "and replay it (steps are rounded to whole replays)")
    ap.add_argument("--stream-rows", choices=["auto", "on", "off"], default="auto",
                    help="pooling loads table rows with the non-temporal hint; auto = only for "
                         "workloads whose ids are drawn uniformly (no reuse for the caches to serve)")
    ap.add_argument("--fuse-mlp", choices=["auto", "on", "off"], default="auto",
                    help="runs of narrow FC layers as one kernel: the library's choice, always, never")
    ap.add_argument("--latency-sweep", action="store_true",
                    help="batch-size sweep with per-batch latency percentiles instead of the "
                         "throughput run (meant for --workload rmc2-large)")
    ap.add_argument("--search", action="store_true",
                    help="gradient search for (instances, batch size) under --sla-ms instead of "
                         "the throughput run; batch sizes from --sweep-batches")
    ap.add_argument("--search-instances", type=int, default=4)
    ap.add_argument("--search-exhaustive", action="store_true",
                    help="with --search: also measure every grid point")
    ap.add_argument("--sweep-batches", default="64,256,1024,4096,16384")
    ap.add_argument("--sweep-iters", type=int, default=200)
    ap.add_argument("--sla-ms", type=float, default=20.0)
    args = ap.parse_args()
    global FUSE_MLP
    FUSE_MLP = args.fuse_mlp
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1")
        return 2
    if args.latency_sweep:
        return latency_sweep(args)
    if args.search:
        return search_mode(args)

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
    global SUSTAINED_RANDOM_TFLOPS
    SUSTAINED = mfma_sustained(torch, binding, dev)
    SUSTAINED_RANDOM_TFLOPS = SUSTAINED["random_operands"]["tflops"]
    streams = pick_concurrent_streams(torch, dev, 4)

    def wants_streaming(wl):
        return args.stream_rows == "on" or (args.stream_rows == "auto" and wl.index_dist[0] == "uniform")

    m, bottom, top = build_model(binding, synth, torch, w, w.batch)
    pm, _, _ = build_model(binding, synth, torch, w, w.batch, share_tables=m, pipeline=True,
                           dense_stream=streams[3], pool_streams=(streams[1], streams[2]))
    for mm in (m, pm):
        mm.set_option(binding.REC_OPT_STREAM_ROWS, int(wants_streaming(w)))
    if args.hot_rows > 0:
        pcdf = synth.zipf_cdf(w.rows, float(w.index_dist[1])) if w.index_dist[0] == "zipf" else None
        hot = synth.profile_hot_rows(w, [900, 901], args.hot_rows, pcdf)
        for mm in (m, pm):
            for t in range(w.num_tables):
                mm.load_hot_rows(t, hot[t])
    log(f"model {w.name}: {w.num_tables} x {w.rows} x {w.emb_dim} {w.table_dtype} resident ({time.time() - t0:.1f} s)")
    host_batches, dev_batches = make_batches(torch, synth, w, args.batches, 0, dev)
    outs = [new_logits(torch, w, w.batch, dev) for _ in range(4)]
    log(f"{args.batches} batches of {w.batch} resident, nnz[0] = {host_batches[0].nnz} ({time.time() - t0:.1f} s)")

    if args.calibration_copy_mib:
        n = args.calibration_copy_mib << 20
        src = torch.full((n,), 1, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Both modes kept up for a few seconds each, before the timed region, so that
    # the K timed steps below see the clocks and caches of a device that has been
    # serving for a while rather than one that idled through the input set-up.
    extra = {}
    if args.sustain_seconds > 0:
        sus = {}
        for label, model in (("pipelined", pm), ("in_order", m)):
            probe = run_steps(torch, model, streams[0], dev_batches, outs, 200)
            n = max(200, int(args.sustain_seconds / (probe / 200)) + 1)
            dt = run_steps(torch, model, streams[0], dev_batches, outs, n)
            sus[label] = {"value": w.batch * n / dt, "unit": "samples/s", "ms_per_step": dt * 1e3 / n,
                          "steps": n, "seconds": dt}
        extra["sustained"] = sus
        log(f"sustained: pipelined {sus['pipelined']['value'] / 1e6:.2f} M, in order "
            f"{sus['in_order']['value'] / 1e6:.2f} M samples/s ({time.time() - t0:.1f} s)")

    # ---- the timed region: exactly K steps, W warm-up steps before it
    timed_model = pm if args.mode == "pipelined" else m
    steps = args.steps
    if args.graph:
        # One replay = one forward over each distinct batch (in the chosen mode).
        per = len(dev_batches)
        glog = [new_logits(torch, w, w.batch, dev) for _ in range(per)]
        with torch.cuda.stream(streams[0]):
            cap = binding.CapturedForward(timed_model, dev_batches, glog)
        steps = max(per, steps // per * per)
        with torch.cuda.stream(streams[0]):
            for _ in range(max(1, args.warmup // per)):
                cap.replay()
        torch.cuda.synchronize()
        t = time.perf_counter()
        with torch.cuda.stream(streams[0]):
            for _ in range(steps // per):
                cap.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t
    else:
        run_steps(torch, timed_model, streams[0], dev_batches, outs, args.warmup)
        st, pos = timed_model.check()
        assert st == binding.REC_OK, (st, pos)
        elapsed = run_steps(torch, timed_model, streams[0], dev_batches, outs, steps, first=args.warmup)
    ms_per_step = elapsed * 1e3 / steps
    value = w.batch * steps / elapsed
    log(f"timed region: {steps} steps, {ms_per_step * 1e3:.1f} us/step, {value / 1e6:.2f} M samples/s ({time.time() - t0:.1f} s)")

    # the other mode over the same K steps
    other = m if timed_model is pm else pm
    run_steps(torch, other, streams[0], dev_batches, outs, args.warmup)
    dt = run_steps(torch, other, streams[0], dev_batches, outs, steps, first=args.warmup)
    extra["in_order" if other is m else "pipelined"] = {
        "value": w.batch * steps / dt, "unit": "samples/s", "ms_per_step": dt * 1e3 / steps, "steps": steps}

    # one batch in flight at a time
    extra["latency_ms"] = latency_profile(torch, np, m, streams[0], dev_batches, outs[0], args.latency_iters)
    extra["latency_ms"]["note"] = "in-order forward of one batch, closed loop, host launch and synchronisation included"

    # every stage of in-order forwards bracketed with HIP events
    stage_avg, pool_ms, used = stage_profile(torch, binding, np, m, streams[0], dev_batches, args.timed_launches)
    this_leg = pool_roofline(np, w, host_batches, used, pool_ms, wants_streaming(w))
    comp = pool_roofline(np, w, host_batches, used, pool_ms, wants_streaming(w), kind="compulsory")
    traffic = this_leg["traffic"]
    pool_detail = dict(this_leg)
    pool_detail.update({
        "algorithmic_gbps": this_leg["achieved"],
        "compulsory_bytes_per_launch": comp["bytes_per_launch"], "compulsory_gbps": comp["achieved"],
        "compulsory_frac_of_hbm_peak": comp["frac"],
        "traffic_source": "rocprofv3 counters of an earlier run of the same kernel source (profiles/), not this run",
        "hbm_frac_by_profiled_traffic": (traffic / (this_leg["avg_launch_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS)
        if traffic else None})
    skewed = w.index_dist[0] == "zipf"
    if skewed:
        pool_detail["note"] = ("skewed ids: the caches serve most rows, so the algorithmic rate may exceed the "
                               "HBM peak; the binding comparison is the uniform-id twin under `roofline`")
        for k in ("frac", "achieved", "bound"):
            pool_detail.pop(k)
        if w.pooling[0] != "fixed" or w.pooling[1] > 1:
            pool_detail["id_repeats"] = repeats_within_chunks(w, host_batches[0])
        extra["roofline_zipf"] = pool_detail
    roofline = None if skewed and w.interaction == "dot" else this_leg

    # the uniform-id twin: the run on which pooling is compared with the HBM peak
    if skewed and w.interaction == "dot":
        wu = w.with_uniform_indices()
        hbu, dbu = make_batches(torch, synth, wu, args.batches, 500, dev)
        m.set_option(binding.REC_OPT_STREAM_ROWS, int(wants_streaming(wu)))
        _, pool_u, used_u = stage_profile(torch, binding, np, m, streams[0], dbu, args.timed_launches)
        st, pos = m.check()
        assert st == binding.REC_OK, (st, pos)
        m.set_option(binding.REC_OPT_STREAM_ROWS, int(wants_streaming(w)))
        roofline = pool_roofline(np, wu, hbu, used_u, pool_u, wants_streaming(wu))
        roofline["note"] = ("uniform-id twin of the headline workload (same shapes, ids uniform): nothing for the "
                            "caches to serve, so algorithmic bytes are HBM bytes")
        del dbu, hbu
    if w.interaction == "concat":
        # Dense-dominated shape: the first Predict-FC layer of all towers is one
        # launch and the longest kernel; its algorithmic work is 2 * B * K * N per tower.
        flops = 2.0 * w.batch * w.top[0] * w.top[1] * w.towers
        tf = flops / (stage_avg["top_first"] * 1e-3) / 1e12
        roofline = {"kernel": "fc_big_kernel (first Predict-FC layer of all towers, one launch)",
                    "bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "flops_per_launch": flops,
                    "avg_launch_ms": stage_avg["top_first"], "launches_timed": args.timed_launches,
                    "pooling": this_leg}
    y = widest_layer_yardstick(torch, w, dev)
    if y:
        extra["library_gemm_yardstick"] = y
    extra["mfma_sustained"] = SUSTAINED
    log(f"stage events done ({time.time() - t0:.1f} s)")

    # Model co-location on the accelerator (Sec. II-B): the same K steps dealt to
    # several in-order instances on streams of their own.
    if args.colocated_leg > 1:
        nc = args.colocated_leg
        cm = [m] + [build_model(binding, synth, torch, w, w.batch, share_tables=m)[0] for _ in range(nc - 1)]
        cs = streams[:nc] if nc <= len(streams) else pick_concurrent_streams(torch, dev, nc)
        cl = [new_logits(torch, w, w.batch, dev) for _ in range(nc)]

        def cstep(i):
            with torch.cuda.stream(cs[i % nc]):
                cm[i % nc].forward(*dev_batches[i % len(dev_batches)], cl[i % nc])
        csteps = max(steps, 200)
        for i in range(args.warmup):
            cstep(i)
        torch.cuda.synchronize()
        tc = time.perf_counter()
        for i in range(csteps):
            cstep(i)
        torch.cuda.synchronize()
        ec = time.perf_counter() - tc
        extra["co_located"] = {"instances": nc, "value": w.batch * csteps / ec, "unit": "samples/s",
                               "ms_per_step": ec * 1e3 / csteps, "steps": csteps}
        for mm in cm[1:]:
            mm.close()

    # What a plain device-to-device copy reaches on this machine (bytes read + written),
    # the practical yardstick beside the published peak.
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    extra["device_copy_gbps"] = 5 * 2 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst

    for mm in (m, pm):
        st, pos = mm.check()
        assert st == binding.REC_OK, (st, pos)
        mm.close()
    del m, pm, dev_batches, outs
    gc.collect()
    torch.cuda.empty_cache()

    # ---- the other configurations, short legs
    if not args.no_other_workloads and args.workload == "rmc2" and not args.uniform and not args.batch:
        others = {}
        for name in ("tiny", "rmc1", "rmc3", "mtwnd"):
            others[name] = short_leg(torch, binding, synth, np, name, args, dev, streams)
            gc.collect()
            torch.cuda.empty_cache()
        wl = synth.WORKLOADS["rmc2-large"]
        free, _ = torch.cuda.mem_get_info()
        need = wl.num_tables * wl.rows * wl.emb_dim * 2 + (8 << 30)
        if free >= need:
            others["rmc2-large"] = sweep_leg(torch, binding, synth, np, wl,
                                             [int(x) for x in args.sweep_batches.split(",")],
                                             args.sweep_iters, args.sla_ms, dev, streams)
        else:
            others["rmc2-large"] = {"skipped": f"needs {need >> 30} GiB of device memory, {free >> 30} GiB free"}
        extra["other_workloads"] = others
        gc.collect()
        torch.cuda.empty_cache()
        log(f"other workloads done ({time.time() - t0:.1f} s)")

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, host_batches[:args.cpu_batches], bottom, top, args.cpu_samples)

    out = {
        "metric": ("samples/sec per GPU + embedding-bag HBM GB/s (% of peak), RMC2-style" if w.interaction == "dot"
                   else "samples/sec per GPU + first Predict-FC layer TFLOP/s (% of bf16 MFMA peak), MT-WnD-style"),
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dtype_string(w), "data": "synthetic",
        "config": {"workload": workload_string(w), "batch": w.batch, "distinct_batches": args.batches,
                   "mode": f"hip graph of {args.mode} forwards" if args.graph else args.mode,
                   "streams": 4 if args.mode == "pipelined" else 1,
                   "hot_rows_per_table": args.hot_rows,
                   "mean_nnz": float(np.mean([b.nnz for b in host_batches]))},
        "roofline": roofline, "cpu_baseline": cpu, "stage_ms": stage_avg, "mlp_mfma": mlp_mfma(w, stage_avg),
    }
    out.update(extra)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
