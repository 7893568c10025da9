"""Checks of the seeded input generators (no model arithmetic involved)."""
import math

import numpy as np

from paper_2203_07424_amd import synth


def test_workload_shapes_follow_the_interaction_width():
    for w in synth.WORKLOADS.values():
        assert w.bottom[0] == w.num_dense
        assert w.interaction == "concat" or w.bottom[-1] == w.emb_dim
        assert w.top[0] == w.interact_width and w.top[-1] == 1
    assert synth.WORKLOADS["mtwnd"].top[0] == 64 + 26 * 64 and synth.WORKLOADS["mtwnd"].towers == 4
    assert synth.WORKLOADS["mtwnd-tiny"].top[0] == 40 + 5 * 32
    assert synth.WORKLOADS["tiny"].top[0] == 68
    assert synth.WORKLOADS["rmc1"].top[0] == 119
    assert synth.WORKLOADS["rmc2"].top[0] == 884
    assert synth.WORKLOADS["rmc3"].top[0] == 87
    assert synth.WORKLOADS["rmc2-large"].top[0] == 1894


def test_splitmix64_first_outputs():
    # First outputs of SplitMix64 seeded with 0, as produced by the public
    # reference implementation of the generator (splitmix64.c, S. Vigna).
    with np.errstate(over="ignore"):
        n = np.arange(3, dtype=np.uint64)
        z = synth._mix64(np.uint64(0) + (n + np.uint64(1)) * synth._GOLDEN)
    assert [int(v) for v in z] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_table_values_range_grid_and_determinism():
    r = np.array([0, 1, 5, 1_999_999, 19_999_999])
    a = synth.table_rows(2203, 3, r, 64, "f32")
    b = synth.table_rows(2203, 3, r, 64, "f32")
    assert a.dtype == np.float32 and a.shape == (5, 64) and np.array_equal(a, b)
    assert (a >= -0.05).all() and (a < 0.05).all()
    assert not np.array_equal(a, synth.table_rows(2203, 4, r, 64, "f32"))
    assert not np.array_equal(a, synth.table_rows(2204, 3, r, 64, "f32"))
    h = synth.table_rows(2203, 3, r, 64, "f16")
    assert h.dtype == np.float16 and np.array_equal(h, a.astype(np.float16))
    # rows are independent of which other rows are asked for
    assert np.array_equal(synth.table_rows(2203, 3, r[2:3], 64, "f32"), a[2:3])
    big = synth.table_rows(2203, 0, np.arange(20000), 32, "f32")
    assert abs(big.mean()) < 2e-4 and abs(big.std() - 0.1 / math.sqrt(12)) < 2e-4


def test_rank_permutation_is_a_bijection():
    for rows in [1, 2, 3, 10, 64, 97, 1000, 2000]:
        a, c = synth.rank_permutation(2203, 1, rows)
        assert math.gcd(a, rows) == 1
        img = (np.arange(rows, dtype=np.int64) * a + c) % rows
        assert np.array_equal(np.sort(img), np.arange(rows))


def test_zipf_head_probability_and_support():
    w = synth.WORKLOADS["rmc2"]
    small = synth.Workload("z", 2, 5000, 8, "f16", 4000, 4, ("fixed", 50), ("zipf", 1.05),
                           (4, 8), (8 + 3, 1))
    cdf = synth.zipf_cdf(small.rows, 1.05)
    H = (np.arange(1, small.rows + 1) ** -1.05).sum()
    assert abs(cdf[0] - 1.0 / H) < 1e-15 and cdf[-1] == 1.0
    lens = synth.draw_lengths(small, 0)
    idx = synth.draw_indices(small, 0, lens)
    assert idx.min() >= 0 and idx.max() < small.rows and idx.size == 2 * 4000 * 50
    n = 4000 * 50
    for t in range(2):
        a, c = synth.rank_permutation(small.seed, t, small.rows)
        hot_row = c % small.rows                  # image of rank 0
        p_hat = (idx[t * n:(t + 1) * n] == hot_row).mean()
        assert abs(p_hat - 1.0 / H) < 4 * math.sqrt((1 / H) / n)
    assert w.index_dist == ("zipf", 1.05)


def test_poisson_lengths_clamped_and_moments():
    w = synth.WORKLOADS["rmc2"].with_batch(512)
    lens = synth.draw_lengths(w, 0)
    assert lens.dtype == np.int32 and lens.size == 40 * 512
    assert lens.min() >= 1 and lens.max() <= 200
    assert abs(lens.mean() - 80.0) < 0.5 and abs(lens.var() - 80.0) < 4.0
    assert np.array_equal(lens, synth.draw_lengths(w, 0))
    assert not np.array_equal(lens, synth.draw_lengths(w, 1))


def test_batch_is_reproducible_and_consistent():
    w = synth.WORKLOADS["tiny"]
    a, b = synth.draw_batch(w, 0), synth.draw_batch(w, 0)
    assert a.dense.tobytes() == b.dense.tobytes() and a.indices.tobytes() == b.indices.tobytes()
    assert a.dense.shape == (256, 13) and a.lengths.sum() == a.nnz == 8 * 256 * 20
    assert a.indices.max() < w.rows and a.indices.min() >= 0
    W, bias = synth.draw_mlp(w, "bottom")[0]
    assert W.shape == (256, 13) and bias.shape == (256,)
    assert abs(W.std() - 13 ** -0.5) < 0.02
    # towers draw from streams of their own; tower 0 is the single-stack stream
    m = synth.WORKLOADS["mtwnd-tiny"]
    t0, t1 = synth.draw_mlp(m, "top", 0), synth.draw_mlp(m, "top", 1)
    assert t0[0][0].shape == (96, 200) and not np.array_equal(t0[0][0], t1[0][0])
    assert np.array_equal(t0[0][0], synth.draw_mlp(m, "top")[0][0])
    assert synth.draw_mlp(synth.WORKLOADS["mtwnd"], "bottom") == []
    one = synth.draw_batch(m, 0)
    assert one.nnz == 5 * 200 and (one.lengths == 1).all()


def test_slice_and_compaction_keep_bag_contents():
    w = synth.Workload("s", 3, 1000, 8, "f16", 16, 4, ("poisson", 6.0, 1, 20), ("zipf", 1.05),
                       (4, 8), (8 + 6, 1))
    batch = synth.draw_batch(w, 2)
    pick = np.array([3, 0, 11])
    sub = synth.slice_samples(w, batch, pick)
    off = np.concatenate([[0], np.cumsum(batch.lengths)])
    soff = np.concatenate([[0], np.cumsum(sub.lengths)])
    for t in range(3):
        for j, b in enumerate(pick):
            want = batch.indices[off[t * 16 + b]:off[t * 16 + b + 1]]
            got = sub.indices[soff[t * 3 + j]:soff[t * 3 + j + 1]]
            assert np.array_equal(want, got)
    assert np.array_equal(sub.dense, batch.dense[pick])
    tabs, cidx = synth.compact_tables(w, sub, 3)
    pos = 0
    per_table = sub.lengths.reshape(3, 3).sum(axis=1)
    for t in range(3):
        n = int(per_table[t])
        want = synth.table_rows(w.seed, t, sub.indices[pos:pos + n], 8, "f16")
        assert np.array_equal(tabs[t][cidx[pos:pos + n]], want)
        pos += n
