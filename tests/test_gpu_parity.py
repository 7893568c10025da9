"""Parity of the HIP path (through the C boundary) against the CPU oracle.

Integer work (offsets, error positions, synthetic table bits) must be bit-exact;
fp32 pooling within 1e-5 relative; bf16 MLP logits within 2e-2 relative of the
exact oracle.  Every test prints what it runs before touching the GPU.
"""
import numpy as np
import pytest
import torch

from oracle import rec_oracle as orc
from paper_2203_07424_amd import synth

import gpu_helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2203_07424_amd import binding as b
    return b


def say(*a):
    print(*a, flush=True)


def small_mlps(g, F, D, T, hidden_b=(24,), hidden_t=(16,)):
    def stack(ws):
        return [((g.standard_normal((ws[i + 1], ws[i])) * ws[i] ** -0.5).astype(np.float32),
                 (g.standard_normal(ws[i + 1]) * ws[i] ** -0.5).astype(np.float32))
                for i in range(len(ws) - 1)]
    return stack((F,) + tuple(hidden_b) + (D,)), stack((D + T * (T + 1) // 2,) + tuple(hidden_t) + (1,))


# ------------------------------------------------------------- generator
@pytest.mark.parametrize("dtype,D,rows", [("f32", 32, 5000), ("f16", 64, 70001), ("f16", 8, 333)])
def test_device_table_fill_matches_host_generator(binding, dtype, D, rows):
    say("fill", dtype, D, rows)
    tdt = torch.float16 if dtype == "f16" else torch.float32
    tab = torch.empty((rows, D), dtype=tdt, device="cuda")
    assert binding.rec_synth_fill_table(tab, 2203, 7) == binding.REC_OK
    torch.cuda.synchronize()
    want = synth.table_rows(2203, 7, np.arange(rows), D, dtype)
    bits = np.uint16 if dtype == "f16" else np.uint32
    got_b, want_b = tab.cpu().numpy().view(bits), want.view(bits)
    bad = np.argwhere(got_b != want_b)
    if bad.size:
        f32 = synth.table_rows(2203, 7, np.arange(rows), D, "f32")
        ex = [(int(r), int(c), hex(got_b[r, c]), hex(want_b[r, c]), float(f32[r, c]).hex())
              for r, c in bad[:8]]
        pytest.fail(f"{len(bad)} of {got_b.size} elements differ, e.g. {ex}")


# ------------------------------------------------------------- S0 + S1
POOL_CASES = [
    # T, R, D, dtype, B, lo, hi
    (3, 1000, 32, np.float32, 37, 0, 50),      # 128-byte rows
    (2, 5000, 64, np.float16, 129, 1, 200),    # 128-byte rows, several id chunks
    (2, 800, 64, np.float32, 65, 0, 130),      # 256-byte rows
    (4, 300, 8, np.float16, 50, 0, 70),        # 16-byte rows: 64 rows per load
    (2, 300, 4, np.float32, 33, 0, 9),         # 16-byte rows
    (1, 200, 256, np.float32, 9, 0, 17),       # 1 KB rows: one row per load
    (2, 100, 128, np.float16, 40, 0, 300),     # long bags
    (5, 2000, 16, np.float32, 1500, 0, 12),    # T*B spans several scan tiles
    (3, 500, 4, np.float32, 100_000, 0, 3),    # 300,000 bags: 147 scan tiles
]


@pytest.mark.parametrize("T,R,D,dtype,B,lo,hi", POOL_CASES)
def test_offsets_bit_exact_and_pooling_within_tolerance(binding, T, R, D, dtype, B, lo, hi):
    say("pool case", T, R, D, dtype.__name__, B, lo, hi)
    g = np.random.default_rng(100 + T * 7 + D)
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(dtype) for _ in range(T)]
    lens = g.integers(lo, hi + 1, T * B).astype(np.int32)
    lens[g.integers(0, T * B, 3)] = 0
    idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
    bottom, top = small_mlps(g, 5, D, T)
    m = H.make_model(binding, tabs, bottom, top, B, int(lens.sum()) + 5, 5)
    batch = synth.Batch(g.standard_normal((B, 5)).astype(np.float32), idx, lens)
    H.run(m, batch)
    assert m.check() == (binding.REC_OK, -1)
    off, rc, _ = orc.offsets(lens)
    assert np.array_equal(m.debug_offsets().cpu().numpy().astype(np.int64), off)
    P, A, nbad, _ = orc.pool(tabs, idx, lens, B, want_abs=True)
    assert nbad == 0
    got = m.debug_pooled().cpu().numpy()
    H.check_pooled(got, P, A)
    # run-to-run determinism: fixed reduction order
    H.run(m, batch)
    assert np.array_equal(got, m.debug_pooled().cpu().numpy())
    m.close()


def test_streaming_row_loads_give_the_same_sums(binding):
    # The non-temporal hint changes where rows are cached, not what is summed.
    say("streaming rows")
    g = np.random.default_rng(61)
    for (T, R, D, dtype, B) in [(3, 2000, 64, np.float16, 300), (2, 500, 32, np.float32, 129), (1, 300, 256, np.float32, 17)]:
        tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(dtype) for _ in range(T)]
        lens = g.integers(0, 150, T * B).astype(np.int32)
        idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
        bottom, top = small_mlps(g, 4, D, T)
        dense = g.standard_normal((B, 4)).astype(np.float32)
        m = H.make_model(binding, tabs, bottom, top, B, idx.size, 4)
        batch = synth.Batch(dense, idx, lens)
        cached = H.run(m, batch)
        pooled_cached = m.debug_pooled().cpu().numpy()
        m.set_option(binding.REC_OPT_STREAM_ROWS, 1)
        streamed = H.run(m, batch)
        assert np.array_equal(pooled_cached, m.debug_pooled().cpu().numpy())
        assert np.array_equal(cached, streamed)
        P, A, nbad, _ = orc.pool(tabs, idx, lens, B, want_abs=True)
        H.check_pooled(m.debug_pooled().cpu().numpy(), P, A)
        assert m.check() == (binding.REC_OK, -1)
        m.close()


@pytest.mark.parametrize("hi,hot", [(150, False), (3, False), (150, True)])
def test_slots_without_a_row_add_nothing_even_next_to_nan(binding, hi, hot):
    # Lanes past the end of a bag and ids outside the table must not pick up any
    # row: row 0, the nearest candidate, holds NaN and infinities here.
    say("no-row slots", hi, hot)
    g = np.random.default_rng(77 + hi)
    for (T, R, D, dtype, B) in [(3, 900, 64, np.float16, 130), (2, 400, 32, np.float32, 67), (2, 300, 8, np.float16, 40)]:
        tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(dtype) for _ in range(T)]
        for tab in tabs:
            tab[0, ::3] = np.nan
            tab[0, 1::3] = np.inf
            tab[0, 2::3] = -np.inf
        lens = g.integers(0, hi + 1, T * B).astype(np.int32)
        idx = g.integers(1, R, int(lens.sum())).astype(np.int32)
        bad_at = g.permutation(idx.size)[:7]
        idx[bad_at] = np.array([R, -1, R + 5, -2 ** 31, 2 ** 31 - 1, R, -7], dtype=np.int32)
        bottom, top = small_mlps(g, 4, D, T)
        m = H.make_model(binding, tabs, bottom, top, B, idx.size, 4)
        if hot:
            for t in range(T):
                m.load_hot_rows(t, g.integers(0, R, 64).astype(np.int32))
        H.run(m, synth.Batch(g.standard_normal((B, 4)).astype(np.float32), idx, lens))
        P, A, nbad, first = orc.pool(tabs, idx, lens, B, want_abs=True)
        assert nbad == 7 and m.check() == (binding.REC_ERR_INDEX_RANGE, first)
        got = m.debug_pooled().cpu().numpy()
        assert np.isfinite(got).all()
        H.check_pooled(got, P, A)
        m.close()


def test_table_beyond_four_gib(binding):
    # Rows past byte 2^32 of a table: 64-bit row addresses, same sums.  The table
    # is zero but for a few hundred rows, so the oracle works on those rows alone.
    say("table > 4 GiB")
    g = np.random.default_rng(91)
    D, R, R2, B, F = 256, 4_400_000, 700, 90, 4          # 1 KiB rows: 4.5 GB
    live = np.unique(np.concatenate([g.integers(1, R, 300), [1, 4194303, 4194304, 4194305, R - 1]]))
    vals = g.uniform(-0.05, 0.05, (live.size, D)).astype(np.float32)
    small = g.uniform(-0.05, 0.05, (R2, D)).astype(np.float32)
    big = torch.zeros((R, D), dtype=torch.float32, device="cuda")
    big[torch.from_numpy(live).cuda()] = torch.from_numpy(vals).cuda()
    big[0] = float("nan")
    lens = g.integers(0, 40, 2 * B).astype(np.int32)
    n0 = int(lens[:B].sum())
    pick = g.integers(0, live.size, n0)
    idx = np.concatenate([live[pick], g.integers(0, R2, int(lens[B:].sum()))]).astype(np.int32)
    compact = np.concatenate([pick, idx[n0:]]).astype(np.int32)   # the same bags on the compacted table
    for pos, bad in [(3, R), (17, -1), (n0 - 1, 2 ** 31 - 1)]:
        idx[pos] = bad
        compact[pos] = -1
    bottom, top = small_mlps(g, F, D, 2)
    m = binding.RecModel(2, D, [R, R2], "f32", F, [F] + [W.shape[0] for W, _ in bottom],
                         [top[0][0].shape[1]] + [W.shape[0] for W, _ in top], B, idx.size)
    m.load_table(0, big)
    m.load_table(1, torch.from_numpy(small).cuda())
    H.load_mlps(binding, m, bottom, top)
    batch = synth.Batch(g.standard_normal((B, F)).astype(np.float32), idx, lens)
    for stream in (0, 1):
        m.set_option(binding.REC_OPT_STREAM_ROWS, stream)
        got_logits = H.run(m, batch)
        assert m.check() == (binding.REC_ERR_INDEX_RANGE, 3)
        P, A, nbad, first = orc.pool([vals, small], compact, lens, B, want_abs=True)
        assert nbad == 3 and first == 3
        got = m.debug_pooled().cpu().numpy()
        assert np.isfinite(got).all()
        H.check_pooled(got, P, A)
        exact = orc.forward(batch.dense, [vals, small], compact, lens, bottom, top)
        H.check_logits(got_logits, exact["logits"])
    m.close()
    del big
    torch.cuda.empty_cache()


def test_pooling_closed_forms_on_device(binding):
    say("pool closed forms")
    g = np.random.default_rng(7)
    T, R, D, B = 2, 4096, 32, 64
    lens = g.integers(0, 90, T * B).astype(np.int32)
    idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
    bottom, top = small_mlps(g, 4, D, T)
    dense = g.standard_normal((B, 4)).astype(np.float32)
    # all-ones tables: pooled value = bag length, exactly
    m = H.make_model(binding, [np.ones((R, D), np.float32)] * T, bottom, top, B, idx.size, 4)
    H.run(m, synth.Batch(dense, idx, lens))
    got = m.debug_pooled().cpu().numpy()
    assert np.array_equal(got, np.repeat(lens.reshape(T, B).T[:, :, None], D, 2).astype(np.float32))
    m.close()
    # row r holds (r mod 2048) + column: sums of small integers are exact in fp32
    tab = ((np.arange(R) % 2048)[:, None] + np.arange(D)[None, :]).astype(np.float32)
    m = H.make_model(binding, [tab] * T, bottom, top, B, idx.size, 4)
    H.run(m, synth.Batch(dense, idx, lens))
    P, _, _, _ = orc.pool([tab] * T, idx, lens, B)
    assert np.array_equal(m.debug_pooled().cpu().numpy().astype(np.float64), P)
    # single-id bags return the row bit for bit (pooling factor 1 = plain lookup)
    ones = np.ones(T * B, np.int32)
    idx1 = g.integers(0, R, T * B).astype(np.int32)
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(np.float32) for _ in range(T)]
    m2 = H.make_model(binding, tabs, bottom, top, B, idx1.size, 4)
    H.run(m2, synth.Batch(dense, idx1, ones))
    got = m2.debug_pooled().cpu().numpy()
    for t in range(T):
        assert np.array_equal(got[:, t, :], tabs[t][idx1[t * B:(t + 1) * B]])
    m.close()
    m2.close()


def test_device_faults_are_reported_not_fatal(binding):
    say("device faults")
    g = np.random.default_rng(8)
    T, R, D, B = 2, 50, 32, 6
    tabs = [g.uniform(-1, 1, (R, D)).astype(np.float32) for _ in range(T)]
    bottom, top = small_mlps(g, 4, D, T)
    dense = g.standard_normal((B, 4)).astype(np.float32)
    lens = np.array([3, 2, 0, 4, 1, 2, 2, 2, 3, 1, 0, 5], dtype=np.int32)
    idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
    m = H.make_model(binding, tabs, bottom, top, 8, 100, 4)
    # ids outside the table: contribute zero, smallest position reported
    bad = idx.copy()
    bad[4] = R
    bad[9] = -3
    H.run(m, synth.Batch(dense, bad, lens))
    P, _, nbad, first = orc.pool(tabs, bad, lens, B)
    assert nbad == 2 and first == 4
    assert m.check() == (binding.REC_ERR_INDEX_RANGE, 4)
    assert np.allclose(m.debug_pooled().cpu().numpy(), P, rtol=1e-6, atol=1e-6)
    assert m.check() == (binding.REC_OK, -1)          # the record was cleared
    # negative length: counts as zero, position reported
    neg = lens.copy()
    neg[3] = -4
    idx2 = g.integers(0, R, int(np.maximum(neg, 0).sum())).astype(np.int32)
    H.run(m, synth.Batch(dense, idx2, neg))
    off, rc, badpos = orc.offsets(neg)
    assert rc == -1 and badpos == 3
    assert m.check() == (binding.REC_ERR_LENGTHS, 3)
    assert np.array_equal(m.debug_offsets().cpu().numpy().astype(np.int64), off)
    # sum(lengths) != nnz: reported, offsets clamped to nnz so nothing past it is read
    short = idx[:-4]
    logits = H.run(m, synth.Batch(dense, short, lens))
    assert m.check() == (binding.REC_ERR_LENGTHS, -1)
    assert np.isfinite(logits).all()
    assert m.debug_offsets().cpu().numpy().max() == short.size
    # host-checkable faults return at once
    d = torch.from_numpy(dense).cuda()
    assert binding.rec_forward(m.handle, d, None, None, B, 5, None) == binding.REC_ERR_ARG
    assert binding.rec_forward(m.handle, d, None, None, 9, 5, None) == binding.REC_ERR_ARG
    assert binding.rec_forward(m.handle, None, None, None, 0, 0, None) == binding.REC_OK
    m.close()


# ------------------------------------------------------------- whole forward
FWD_CASES = [
    # T, R, D, dtype, B, F, hidden_b, hidden_t
    (3, 500, 32, np.float32, 70, 13, (40,), (24,)),         # ragged everything
    (8, 300, 32, np.float16, 1, 5, (64, 32), (64,)),        # a single sample
    (10, 400, 64, np.float32, 130, 256, (128,), (256, 64)),  # RMC1-like stacks
    (6, 200, 16, np.float16, 257, 100, (), ()),             # one-layer stacks
    (12, 150, 64, np.float16, 200, 64, (256, 128), (512, 128)),
]


@pytest.mark.parametrize("T,R,D,dtype,B,F,hb,ht", FWD_CASES)
def test_forward_every_stage_against_oracle(binding, T, R, D, dtype, B, F, hb, ht):
    say("forward case", T, R, D, dtype.__name__, B, F, hb, ht)
    g = np.random.default_rng(200 + T + B)
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(dtype) for _ in range(T)]
    lens = g.integers(0, 60, T * B).astype(np.int32)
    idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
    bottom, top = small_mlps(g, F, D, T, hb, ht)
    dense = g.standard_normal((B, F)).astype(np.float32)
    m = H.make_model(binding, tabs, bottom, top, B + 3, idx.size, F)
    logits = H.run(m, synth.Batch(dense, idx, lens))
    assert m.check() == (binding.REC_OK, -1)
    exact = orc.forward(dense, tabs, idx, lens, bottom, top, orc.EXACT)
    mirror = orc.forward(dense, tabs, idx, lens, bottom, top, orc.BF16_MIRROR)
    # Bottom-FC output (fp32 on the device)
    x0 = m.debug_bottom_out().cpu().numpy().astype(np.float64)
    scale = np.abs(mirror["bottom_out"]).max() + 1e-30
    assert np.abs(x0 - mirror["bottom_out"]).max() <= 2e-3 * scale
    assert np.abs(x0 - exact["bottom_out"]).max() <= 2e-2 * scale
    # interaction (bf16 on the device): compare with the oracle's formula on the
    # device's own fp32 inputs, within one bf16 rounding
    z = m.debug_interact().float().cpu().numpy().astype(np.float64)
    width = D + T * (T + 1) // 2
    assert not z[:, width:].any()
    P = m.debug_pooled().cpu().numpy().astype(np.float64)
    zo = orc.interact(x0, P)
    assert np.abs(z[:, :width] - zo).max() <= 2.0 ** -8 * np.abs(zo).max() + 1e-30
    # per term: the bf16 narrowing of the output (2^-9 relative, 2^-8 allowed) plus the
    # device's dot product, good to 2^-16 of sum |x_i y_i| (operands split into two
    # bf16 halves on the matrix cores; 2^-14 allowed)
    scale = orc.interact(np.abs(x0), np.abs(P))
    scale[:, :D] = 0.0
    assert (np.abs(z[:, :width] - zo) <= 2.0 ** -8 * np.abs(zo) + 2.0 ** -14 * scale + 1e-30).all()
    # logits
    H.check_logits(logits, exact["logits"], mirror["logits"])
    m.close()


@pytest.mark.parametrize("D,dtype,n_hot", [(64, np.float16, 128), (32, np.float32, 100), (64, np.float32, 37),
                                            (8, np.float16, 1024), (128, np.float16, 120)])
def test_hot_row_cache_gives_the_same_pooling(binding, D, dtype, n_hot):
    """Hot rows served from LDS: same sums as the oracle, with lists that hold
    duplicates, ids outside the table and ids nobody asks for; one table has
    no list at all; faults in the looked-up ids are still reported."""
    say("hot rows", D, dtype.__name__, n_hot)
    g = np.random.default_rng(51 + D + n_hot)
    T, R, B, F = 4, 3000, 300, 8
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(dtype) for _ in range(T)]
    bottom, top = small_mlps(g, F, D, T)
    # skewed ids so that the lists matter: half of the lookups go to 150 rows
    lens = g.integers(0, 150, T * B).astype(np.int32)
    nnz = int(lens.sum())
    hot_pool = g.permutation(R)[:150]
    idx = np.where(g.random(nnz) < 0.5, hot_pool[g.integers(0, 150, nnz)], g.integers(0, R, nnz)).astype(np.int32)
    m = H.make_model(binding, tabs, bottom, top, B, nnz, F)
    batch = synth.Batch(g.standard_normal((B, F)).astype(np.float32), idx, lens)
    plain = H.run(m, batch)
    plain_pooled = m.debug_pooled().cpu().numpy()
    for t in range(T - 1):                                   # the last table keeps no list
        ids = hot_pool[g.permutation(150)[:min(n_hot, 150)]].astype(np.int32)
        extra = np.array([ids[0], R, -5, R + 7, ids[-1]], dtype=np.int32)      # duplicates and bad ids
        ids = np.concatenate([ids, extra, g.integers(0, R, max(0, n_hot - ids.size - 5)).astype(np.int32)])[:n_hot]
        m.load_hot_rows(t, ids)
    hot = H.run(m, batch)
    assert m.check() == (binding.REC_OK, -1)
    P, A, nbad, _ = orc.pool(tabs, idx, lens, B, want_abs=True)
    got = m.debug_pooled().cpu().numpy()
    H.check_pooled(got, P, A)
    H.check_pooled(plain_pooled, P, A)
    off, _, _ = orc.offsets(lens)
    assert np.array_equal(m.debug_offsets().cpu().numpy().astype(np.int64), off)
    exact = orc.forward(batch.dense, tabs, idx, lens, bottom, top)
    mirror = orc.forward(batch.dense, tabs, idx, lens, bottom, top, orc.BF16_MIRROR)
    H.check_logits(hot, exact["logits"], mirror["logits"])
    H.run(m, batch)                                          # reproducible
    assert np.array_equal(got, m.debug_pooled().cpu().numpy())
    # faults among the looked-up ids are still found, also next to hot ids
    bad = idx.copy()
    bad[11] = R + 3
    bad[5000] = -1
    H.run(m, synth.Batch(batch.dense, bad, lens))
    Pb, _, nb, first = orc.pool(tabs, bad, lens, B)
    assert nb == 2 and m.check() == (binding.REC_ERR_INDEX_RANGE, first)
    assert np.allclose(m.debug_pooled().cpu().numpy(), Pb, rtol=1e-5, atol=1e-6)
    # removing the lists returns to the plain kernel, bit for bit
    for t in range(T):
        m.load_hot_rows(t, None)
    again = H.run(m, batch)
    assert np.array_equal(again, plain) and np.array_equal(m.debug_pooled().cpu().numpy(), plain_pooled)
    m.close()


def test_hot_row_list_limits(binding):
    say("hot row limits")
    g = np.random.default_rng(5)
    tabs = [g.uniform(-1, 1, (50, 64)).astype(np.float32)]          # 256-byte rows
    bottom, top = small_mlps(g, 4, 64, 1)
    m = H.make_model(binding, tabs, bottom, top, 4, 100, 4)
    ids = torch.arange(0, 50, dtype=torch.int32, device="cuda")
    assert binding.rec_load_hot_rows(m.handle, 0, ids) == binding.REC_OK
    assert binding.rec_load_hot_rows(m.handle, 1, ids) == binding.REC_ERR_ARG          # table id
    big = torch.zeros(1025, dtype=torch.int32, device="cuda")
    assert binding.rec_load_hot_rows(m.handle, 0, big) == binding.REC_ERR_ARG          # > REC_MAX_HOT_ROWS
    assert binding.rec_load_hot_rows(m.handle, 0, big[:512]) == binding.REC_ERR_ARG    # 128 KB of rows: no fit
    assert binding.rec_load_hot_rows(m.handle, 0, None) == binding.REC_OK
    m.close()


def test_dense_overlap_does_not_change_results(binding):
    """Bottom-FC on the side stream or in order: same kernels, same bits; and a
    run of back-to-back forwards with different inputs keeps them apart."""
    say("overlap on/off")
    g = np.random.default_rng(31)
    T, R, D, B, F = 6, 300, 32, 333, 40
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(np.float16) for _ in range(T)]
    bottom, top = small_mlps(g, F, D, T, (128, 64), (256, 128))
    m = H.make_model(binding, tabs, bottom, top, B, 60 * T * B, F)
    batches = []
    for _ in range(3):
        lens = g.integers(0, 60, T * B).astype(np.int32)
        idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
        batches.append(synth.Batch(g.standard_normal((B, F)).astype(np.float32), idx, lens))
    dev = [(torch.from_numpy(b.dense).cuda(), torch.from_numpy(b.indices).cuda(),
            torch.from_numpy(b.lengths).cuda()) for b in batches]
    outs = {}
    for overlap in (1, 0):
        m.set_option(binding.REC_OPT_OVERLAP_DENSE, overlap)
        res = [torch.empty(B, dtype=torch.float32, device="cuda") for _ in range(12)]
        for i in range(12):                       # no synchronisation in between
            d, ix, ln = dev[i % 3]
            m.forward(d, ix, ln, res[i])
        torch.cuda.synchronize()
        outs[overlap] = [r.cpu().numpy() for r in res]
        assert m.check() == (binding.REC_OK, -1)
    for i in range(12):
        assert np.array_equal(outs[1][i], outs[0][i])
        assert np.array_equal(outs[1][i], outs[1][i % 3])
    for i in range(3):
        b = batches[i]
        exact = orc.forward(b.dense, tabs, b.indices, b.lengths, bottom, top)
        mirror = orc.forward(b.dense, tabs, b.indices, b.lengths, bottom, top, orc.BF16_MIRROR)
        H.check_logits(outs[1][i], exact["logits"], mirror["logits"])
    m.close()


def test_graph_replays_match_eager_forwards(binding):
    """A recorded forward is replayed several times with eager work and
    synchronisations in between; every replay must give the eager bits, also
    after the input buffers were refreshed in place."""
    say("graph replay")
    g = np.random.default_rng(41)
    T, R, D, B, F = 5, 400, 32, 190, 24
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(np.float32) for _ in range(T)]
    bottom, top = small_mlps(g, F, D, T, (64,), (128, 64))
    L = 12                                              # fixed lengths: nnz stays the same
    m = H.make_model(binding, tabs, bottom, top, B, L * T * B, F)

    def draw():
        lens = np.full(T * B, L, np.int32)
        idx = g.integers(0, R, L * T * B).astype(np.int32)
        return synth.Batch(g.standard_normal((B, F)).astype(np.float32), idx, lens)
    first = draw()
    bufs = (torch.from_numpy(first.dense).cuda(), torch.from_numpy(first.indices).cuda(),
            torch.from_numpy(first.lengths).cuda())
    out = torch.empty(B, dtype=torch.float32, device="cuda")
    cap = binding.CapturedForward(m, [bufs], [out])
    scratch = torch.zeros(1 << 20, device="cuda")
    for rep in range(5):
        b = first if rep == 0 else draw()
        bufs[0].copy_(torch.from_numpy(b.dense))
        bufs[1].copy_(torch.from_numpy(b.indices))
        out.zero_()
        cap.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy().copy()
        scratch.add_(1.0)                               # unrelated eager work between replays
        eager = H.run(m, b)
        assert np.array_equal(got, eager), rep
        assert m.check() == (binding.REC_OK, -1)
    exact = orc.forward(b.dense, tabs, b.indices, b.lengths, bottom, top)
    mirror = orc.forward(b.dense, tabs, b.indices, b.lengths, bottom, top, orc.BF16_MIRROR)
    H.check_logits(got, exact["logits"], mirror["logits"])
    m.close()


def test_forward_hand_worked_example_is_exact_on_device(binding):
    import json, os
    say("hand example")
    with open(os.path.join(os.path.dirname(__file__), "golden", "hand_example.json")) as f:
        ex = json.load(f)
    # D = 2 rows are 8 bytes, below the 16-byte gather unit: widen to D = 4 with zero columns,
    # which adds zero terms to every dot product.
    tabs = [np.pad(np.array(t, np.float32), ((0, 0), (0, 2))) for t in ex["tables"]]
    bW = np.pad(np.array(ex["bottom"][0]["W"], np.float32), ((0, 2), (0, 0)))
    bb = np.array(ex["bottom"][0]["b"] + [-1.0, -1.0], np.float32)       # ReLU(-1 + ..) = 0 here
    bW[2:] = 0
    t0W = np.array(ex["top"][0]["W"], np.float32)
    t0W = np.concatenate([t0W[:, :2], np.zeros((2, 2), np.float32), t0W[:, 2:]], axis=1)
    top = [(t0W, np.array(ex["top"][0]["b"], np.float32)),
           (np.array(ex["top"][1]["W"], np.float32), np.array(ex["top"][1]["b"], np.float32))]
    m = H.make_model(binding, tabs, [(bW, bb)], top, 2, 5, 2)
    batch = synth.Batch(np.array(ex["dense"], np.float32), np.array(ex["indices"], np.int32),
                        np.array(ex["lengths_table_major"], np.int32))
    logits = H.run(m, batch)
    assert m.debug_offsets().cpu().numpy().tolist() == ex["expect"]["offsets"]
    assert m.debug_pooled().cpu().numpy()[:, :, :2].tolist() == ex["expect"]["pooled"]
    assert logits.tolist() == ex["expect"]["logits"]
    m.close()


def test_tiny_workload_full_batch(binding):
    w = synth.WORKLOADS["tiny"]
    say("tiny workload, full batch")
    m, bottom, top = H.make_workload_model(binding, w)
    batch = synth.draw_batch(w, 0)
    logits = H.run(m, batch)
    assert m.check() == (binding.REC_OK, -1)
    tabs = [synth.full_table(w, t) for t in range(w.num_tables)]
    exact = orc.forward(batch.dense, tabs, batch.indices, batch.lengths, bottom, top)
    mirror = orc.forward(batch.dense, tabs, batch.indices, batch.lengths, bottom, top, orc.BF16_MIRROR)
    P, A, _, _ = orc.pool(tabs, batch.indices, batch.lengths, w.batch, want_abs=True)
    H.check_pooled(m.debug_pooled().cpu().numpy(), P, A)
    H.check_logits(logits, exact["logits"], mirror["logits"])
    m.close()


# ------------------------------------------------------------- full-size workloads
# Device and bf16 mirror narrow the same values, but from slightly different
# sums (fp32 and split-bf16 accumulation against fp64), so a few per cent of the
# narrowed interaction terms land on the other side of a bf16 rounding boundary
# (one unit in the last place, 2^-8 of the term); over a whole 4096-batch the
# worst sample collects a little more of that than the 5e-3 small shapes use.
WHOLE_BATCH_MIRROR_RTOL = 1e-2


def whole_batch_check(binding, m, w, batch, logits, bottom, top, label):
    """Every sample of a full-size batch against the oracle: offsets bit for bit,
    pooled sums and logits to the bars of gpu_helpers."""
    assert m.check() == (binding.REC_OK, -1)
    off = m.debug_offsets().cpu().numpy()
    assert off[0] == 0 and off[-1] == batch.nnz
    assert np.array_equal(np.diff(off.astype(np.int64)), batch.lengths)
    exact, mirror, P, A = H.oracle_on_batch(w, batch, bottom, top)
    cols = (logits.reshape(w.batch, -1), exact["logits"].reshape(w.batch, -1),
            mirror["logits"].reshape(w.batch, -1))
    for k in range(cols[0].shape[1]):
        re, rm = H.per_sample_ratio(cols[0][:, k], cols[1][:, k]), H.per_sample_ratio(cols[0][:, k], cols[2][:, k])
        say(f"{label} tower {k}: per-sample |g-o| / max(|o|, rms) vs the exact oracle: median {np.median(re):.2e} "
            f"p99 {np.percentile(re, 99):.2e} worst {re.max():.2e}, {(re > H.LOGIT_RTOL).sum()} of {w.batch} "
            f"beyond 2e-2; vs the bf16 mirror: median {np.median(rm):.2e} p99 {np.percentile(rm, 99):.2e} "
            f"worst {rm.max():.2e}")
    if w.interaction == "dot":
        H.check_pooled(m.debug_pooled().cpu().numpy(), P, A)
    H.check_logits(logits, exact["logits"], mirror["logits"], mirror_rtol=WHOLE_BATCH_MIRROR_RTOL)
    # Per sample, |g - o| <= 2e-2 max(|o|, rms) against the exact oracle, except
    # where bf16 operands themselves (the oracle's mirror: same narrowing points,
    # fp64 sums, no device involved) already leave the sample beyond that: one
    # sample in a few thousand does, by a few per cent of the bound.
    for k in range(cols[0].shape[1]):
        re = H.per_sample_ratio(cols[0][:, k], cols[1][:, k])
        rme = H.per_sample_ratio(cols[2][:, k], cols[1][:, k])
        say(f"{label} tower {k}: the mirror itself is beyond 2e-2 of the exact oracle on {(rme > H.LOGIT_RTOL).sum()} "
            f"samples (worst {rme.max():.2e})")
        assert (re <= np.maximum(H.LOGIT_RTOL, rme + 2e-3)).all(), (k, float(re.max()))
        assert (re > H.LOGIT_RTOL).sum() <= max(1, w.batch // 1000), int((re > H.LOGIT_RTOL).sum())


@pytest.mark.parametrize("name,uniform", [("rmc3", False), ("rmc1", False), ("rmc2", False), ("rmc2", True)])
def test_full_size_workload_whole_batch_against_oracle(binding, name, uniform):
    """The named workload at its full size, in the launch configuration the
    benchmark times (uniform ids: row loads with the non-temporal hint, the
    leg the HBM figure is quoted on); the oracle recomputes EVERY sample."""
    w = synth.WORKLOADS[name]
    if uniform:
        w = w.with_uniform_indices()
    say("full-size workload, whole batch", w.name)
    m, bottom, top = H.make_workload_model(binding, w)
    m.set_option(binding.REC_OPT_STREAM_ROWS, int(w.index_dist[0] == "uniform"))
    batch = synth.draw_batch(w, 0)
    logits = H.run(m, batch)
    whole_batch_check(binding, m, w, batch, logits, bottom, top, w.name)
    m.close()
    torch.cuda.empty_cache()


def test_co_located_instances_whole_batch_against_oracle(binding):
    """Two instances sharing the tables, each on a stream of its own, forwards
    interleaved without synchronisation (the benchmark's co-located leg): both
    logits buffers against the oracle, and bit-equal to a forward run alone."""
    w = synth.WORKLOADS["rmc2"]
    say("co-located instances", w.name)
    m0, bottom, top = H.make_workload_model(binding, w)
    m1, _, _ = H.make_workload_model(binding, w, share_tables=m0)
    models, streams = [m0, m1], [torch.cuda.Stream(), torch.cuda.Stream()]
    batches = [synth.draw_batch(w, 10 + i) for i in range(2)]
    dev = [(torch.from_numpy(b.dense).cuda(), torch.from_numpy(b.indices).cuda(),
            torch.from_numpy(b.lengths).cuda()) for b in batches]
    alone = [H.run(m0, b) for b in batches]
    outs = [[torch.empty(w.batch, dtype=torch.float32, device="cuda") for _ in range(2)] for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(3):                            # instance k takes batch (rep + k) % 2
        for k in range(2):
            with torch.cuda.stream(streams[k]):
                models[k].forward(*dev[(rep + k) % 2], outs[k][(rep + k) % 2])
    torch.cuda.synchronize()
    for k in range(2):
        assert models[k].check() == (binding.REC_OK, -1)
        for j in range(2):
            assert np.array_equal(outs[k][j].cpu().numpy(), alone[j]), (k, j)
    for j in range(2):
        exact, mirror, _, _ = H.oracle_on_batch(w, batches[j], bottom, top)
        H.check_logits(alone[j], exact["logits"], mirror["logits"], mirror_rtol=WHOLE_BATCH_MIRROR_RTOL)
    m1.close()
    m0.close()
    torch.cuda.empty_cache()


def test_forward_rejects_buffers_smaller_than_the_call_says(binding):
    """The C boundary sees pointers only, so the binding checks sizes before the
    call: a [B] logits buffer for a model with several towers (which once let the
    device write past it), short lengths, short dense.  Nothing is enqueued."""
    say("undersized buffers")
    w = synth.WORKLOADS["mtwnd-tiny"]
    m, _, _ = H.make_workload_model(binding, w)
    batch = synth.draw_batch(w, 0)
    d, i, l = (torch.from_numpy(x).cuda() for x in (batch.dense, batch.indices, batch.lengths))
    B = w.batch
    with pytest.raises(ValueError):
        m.forward(d, i, l, torch.empty(B, dtype=torch.float32, device="cuda"))          # needs [B][3]
    with pytest.raises(ValueError):
        m.forward(d, i, l[:-1].contiguous())
    with pytest.raises(ValueError):
        m.forward(d[:, :-1].contiguous(), i, l)
    with pytest.raises(ValueError):
        m.forward(d, i.to(torch.int64), l)
    with pytest.raises(ValueError):
        m.forward(d, i, l, torch.empty((B, w.towers), dtype=torch.float32))               # host tensor
    out = m.forward(d, i, l, torch.empty((B, w.towers), dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    assert m.check() == (binding.REC_OK, -1) and torch.isfinite(out).all()
    m.close()


def test_large_capacity_variant_sampled_against_oracle(binding):
    """154 GB of tables: rows sit beyond 2 GiB inside a table, so this is the
    case that needs 64-bit row addressing.  Skipped where the device is smaller.
    B = 512 and B = 4096 (a point of the benchmark's latency sweep, all samples
    checked) on one resident model."""
    import gc
    w0 = synth.WORKLOADS["rmc2-large"]
    gc.collect()
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    need = w0.num_tables * w0.rows * w0.emb_dim * 2 + (8 << 30)
    if free < need:
        pytest.skip(f"needs {need >> 30} GiB of device memory, {free >> 30} GiB free")
    m, bottom, top = H.make_workload_model(binding, w0, max_batch=4096)
    cdf = synth.zipf_cdf(w0.rows, float(w0.index_dist[1]))
    for B in (512, 4096):
        w = w0.with_batch(B)
        say("large-capacity workload, batch", w.batch)
        batch = synth.draw_batch(w, 0, cdf)
        assert batch.indices.max() > (1 << 24)          # byte offsets beyond 2^31 are exercised
        logits = H.run(m, batch)
        if B == 4096:
            whole_batch_check(binding, m, w, batch, logits, bottom, top, w.name)
            # the sweep's pipelined leg: the same batch six times through the pipelined
            # model on four streams, bit-equal to in-order forwards with the same launches
            say("large-capacity workload, pipelined")
            streams = [torch.cuda.Stream() for _ in range(4)]
            pm, _, _ = H.make_workload_model(binding, w0, max_batch=4096, share_tables=m, pipeline=True,
                                             dense_stream=streams[3], pool_streams=(streams[1], streams[2]))
            for mm in (m, pm):
                mm.set_option(binding.REC_OPT_FUSE_MLP, 0)
            want = H.run(m, batch)
            d = [torch.from_numpy(a).cuda() for a in (batch.dense, batch.indices, batch.lengths)]
            outs = [torch.full((B,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(6)]
            torch.cuda.synchronize()
            with torch.cuda.stream(streams[0]):
                for o in outs:
                    pm.forward(*d, o)
                pm.drain()
            streams[0].synchronize()
            assert pm.check() == (binding.REC_OK, -1)
            for i, o in enumerate(outs):
                assert np.array_equal(o.cpu().numpy(), want), i
            pm.close()
            m.set_option(binding.REC_OPT_FUSE_MLP, 1)
            continue
        assert m.check() == (binding.REC_OK, -1)
        pick = np.array([0, 1, 255, 256, B - 2, B - 1])
        exact = H.oracle_on_slice(w, batch, pick, bottom, top)
        mirror = H.oracle_on_slice(w, batch, pick, bottom, top, orc.BF16_MIRROR)
        pooled = m.debug_pooled()[torch.from_numpy(pick).cuda()].cpu().numpy()
        H.check_pooled(pooled, exact["pooled"], exact["abs_sum"])
        H.check_logits(logits[pick], exact["logits"], mirror["logits"])
    m.close()
    del m
    gc.collect()
    torch.cuda.empty_cache()


def test_gradient_search_on_measured_throughput(binding):
    """Algorithm 1 driven by real measurements of the forward pass: every move
    of the walk raises throughput within the SLA, and the end point is (within
    measurement noise) the best in-bound point of the fully measured grid."""
    from oracle import search_oracle as so
    from paper_2203_07424_amd import scheduler
    say("gradient search on measured points")
    w0 = synth.WORKLOADS["tiny"]
    sizes, counts = [64, 512, 4096], [1, 2, 3]
    m0, _, _ = H.make_workload_model(binding, w0, max_batch=max(sizes))
    models = [m0]
    for _ in counts[1:]:
        m = binding.RecModel(w0.num_tables, w0.emb_dim, [w0.rows] * w0.num_tables, w0.table_dtype,
                             w0.num_dense, list(w0.bottom), list(w0.top), max(sizes),
                             max(sizes) * w0.num_tables * 20)
        for t in range(w0.num_tables):
            m.load_table(t, m0.tables[t])
        H.load_mlps(binding, m, synth.draw_mlp(w0, "bottom"), synth.draw_mlp(w0, "top"))
        models.append(m)
    streams = [torch.cuda.Stream() for _ in counts]
    data = {}
    for B in sizes:
        b = synth.draw_batch(w0.with_batch(B), 7)
        outs = [torch.empty(B, dtype=torch.float32, device="cuda") for _ in counts]
        data[B] = [(torch.from_numpy(b.dense).cuda(), torch.from_numpy(b.indices).cuda(),
                    torch.from_numpy(b.lengths).cuda(), outs)]
    memo = {}

    def measure(m, d):
        if (m, d) not in memo:
            memo[(m, d)] = scheduler.measure_point(models, streams, data, m, d, rounds=30, warmup=5)
        return memo[(m, d)]
    sla = 50.0
    res = scheduler.search(measure, counts, sizes, sla)
    assert res.instances is not None and res.path[0] == (1, 64)
    for p, q in zip(res.path, res.path[1:]):
        assert memo[q].qps > memo[p].qps and memo[q].latency_ms < sla
    tab = lambda i, j: (measure(counts[i], sizes[j]).qps, measure(counts[i], sizes[j]).latency_ms, 0.0)
    best, best_qps = so.exhaustive(tab, len(counts), len(sizes), sla)
    got, path = so.algorithm1(tab, len(counts), len(sizes), sla)      # same table, oracle's walk
    assert [(counts[i], sizes[j]) for i, j in path] == res.path
    assert res.measurement.qps >= 0.85 * best_qps                     # convexity, up to noise
    for m in models:
        assert m.check() == (binding.REC_OK, -1)
        m.close()


@pytest.mark.parametrize("F,B", [(200, 3000), (203, 3000), (512, 3100)])
def test_wide_bottom_layer_on_fp32_input(binding, F, B):
    # A first Bottom-FC layer wide enough, on a batch large enough, for the
    # 128 x 128 double-buffered tile that reads the fp32 dense input directly:
    # F = 200 ends inside a k-tile (the rest must count as zero), F = 203 is not a
    # multiple of 8 (the general kernel takes it), B is not a multiple of the tile.
    say("wide bottom", F, B)
    g = np.random.default_rng(300 + F)
    T, R, D = 3, 200, 32
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(np.float32) for _ in range(T)]
    lens = g.integers(0, 6, T * B).astype(np.int32)
    idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
    bottom, top = small_mlps(g, F, D, T, (1024,), (64,))
    dense = g.standard_normal((B, F)).astype(np.float32)
    m = H.make_model(binding, tabs, bottom, top, B, idx.size, F)
    logits = H.run(m, synth.Batch(dense, idx, lens))
    assert m.check() == (binding.REC_OK, -1)
    exact = orc.forward(dense, tabs, idx, lens, bottom, top, orc.EXACT)
    mirror = orc.forward(dense, tabs, idx, lens, bottom, top, orc.BF16_MIRROR)
    x0 = m.debug_bottom_out().cpu().numpy().astype(np.float64)
    scale = np.abs(mirror["bottom_out"]).max() + 1e-30
    assert np.abs(x0 - mirror["bottom_out"]).max() <= 2e-3 * scale
    H.check_logits(logits, exact["logits"], mirror["logits"])
    m.close()


def test_matrix_rate_probe_runs(binding):
    """The measurement helper behind bench.py's mfma_sustained: both operand kinds run and leave a finite checksum."""
    say("matrix-rate probe")
    sink = torch.full((1,), float("nan"), device="cuda")
    for rnd in (False, True):
        assert binding.rec_probe_mfma(rnd, 64, 50, sink) == binding.REC_OK
        torch.cuda.synchronize()
        assert torch.isfinite(sink).all()
    # constant operands: every product is 1, 16 per instruction, 4 instructions per accumulator and iteration
    assert binding.rec_probe_mfma(False, 8, 10, sink) == binding.REC_OK
    torch.cuda.synchronize()
    assert sink.item() == 8 * 10 * 4 * 16.0
