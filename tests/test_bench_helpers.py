"""Host-side arithmetic of bench.py (no GPU): the byte counts behind the
roofline figures and the id-repeat statistic, on inputs small enough to count
by hand."""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import bench  # noqa: E402
from paper_2203_07424_amd import synth  # noqa: E402


def hand_workload(**kw):
    base = dict(name="hand", num_tables=2, rows=100, emb_dim=8, table_dtype="f16", batch=2, num_dense=4,
                pooling=("poisson", 3.0, 1, 200), index_dist=("zipf", 1.05), bottom=(4, 8), top=(11, 1))
    base.update(kw)
    return synth.Workload(**base)


def test_algorithmic_and_compulsory_pool_bytes_by_hand():
    w = hand_workload()
    # table-major bags: (t0,b0) (t0,b1) (t1,b0) (t1,b1)
    lengths = np.array([3, 1, 2, 2], dtype=np.int32)
    ids = np.array([5, 5, 7,  9,  5, 5,  1, 2], dtype=np.int32)
    b = synth.Batch(np.zeros((2, 4), np.float32), ids, lengths)
    row = 8 * 2                                   # fp16 rows of 8
    # rows gathered + ids + offsets (bags + 1) + pooled vectors written (fp32)
    assert bench.algorithmic_pool_bytes(w, b) == 8 * row + 8 * 4 + 5 * 4 + 4 * 8 * 4
    # distinct rows per table: {5, 7, 9} and {5, 1, 2}
    assert bench.compulsory_pool_bytes(w, b) == 6 * row + 8 * 4 + 5 * 4 + 4 * 8 * 4
    # concatenation model: pooled vectors leave as bf16
    wc = hand_workload(interaction="concat", top=(8 + 2 * 8, 1))
    assert bench.algorithmic_pool_bytes(wc, b) == 8 * row + 8 * 4 + 5 * 4 + 4 * 8 * 2
    # fp32 tables
    wf = hand_workload(table_dtype="f32")
    assert bench.algorithmic_pool_bytes(wf, b) == 8 * 32 + 8 * 4 + 5 * 4 + 4 * 8 * 4


def test_id_repeats_within_chunks_by_hand():
    w = hand_workload(num_tables=1, batch=2)
    # bag 0: 70 ids = a chunk of 64 and a chunk of 6; bag 1: 9 ids
    bag0 = np.concatenate([np.arange(60), [0, 0, 1, 59],      # chunk 0: 60 distinct + 4 repeats
                           [0, 100, 100, 101, 102, 103]])     # chunk 1: 5 distinct + 1 repeat (0 is new here)
    bag1 = np.array([7, 7, 7, 7, 7, 7, 7, 7, 8])              # 2 distinct + 7 repeats
    lengths = np.array([70, 9], dtype=np.int32)
    ids = np.concatenate([bag0, bag1]).astype(np.int32)
    r = bench.repeats_within_chunks(w, synth.Batch(np.zeros((2, 4), np.float32), ids, lengths))
    assert np.isclose(r["lookups_repeating_an_id_of_their_chunk"], (4 + 1 + 7) / 79)
    # wave-wide loads of 8 rows: 8 + 1 + 2 = 11 as is; distinct ids need 8 + 1 + 1 = 10
    assert np.isclose(r["wave_wide_row_loads_saved"], 1 - 10 / 11)
    # no repeats at all
    r = bench.repeats_within_chunks(w, synth.Batch(np.zeros((2, 4), np.float32), np.arange(79, dtype=np.int32), lengths))
    assert r["lookups_repeating_an_id_of_their_chunk"] == 0.0 and r["wave_wide_row_loads_saved"] == 0.0


def test_mlp_flops_and_stage_filter():
    w = synth.WORKLOADS["rmc2"]
    avg = {"bottom_first": 0.0, "bottom_rest": 0.0, "top_first": 0.010, "top_rest": 0.005}
    out = bench.mlp_mfma(w, avg)
    assert set(out) == {"top_first", "top_rest"}             # stages without an interval of their own are left out
    f = 2.0 * w.batch * w.top[0] * w.top[1]
    assert np.isclose(out["top_first"]["gflop"], f / 1e9)
    assert np.isclose(out["top_first"]["tflops"], f / 10e-6 / 1e12)
    assert np.isclose(out["top_first"]["frac_of_bf16_peak"], out["top_first"]["tflops"] / 2500.0)
    rest = sum(2.0 * w.batch * w.top[i] * w.top[i + 1] for i in range(1, len(w.top) - 1))
    assert np.isclose(out["top_rest"]["gflop"], rest / 1e9)


def test_strings_name_the_workload_and_the_arithmetic():
    w = synth.WORKLOADS["mtwnd"]
    assert "4 towers" in bench.workload_string(w) and "concatenation" in bench.workload_string(w)
    assert "interaction" not in bench.dtype_string(w)
    assert "two bf16 planes" in bench.dtype_string(synth.WORKLOADS["rmc2"])
