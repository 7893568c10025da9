"""Pins of the CPU oracle against what the definitions and mathematics fix.

The paper prints no worked forward pass, so the oracle is pinned by: integer
identities, special cases that reduce to a table row or a count, closed
forms, numpy / torch library routines in fp64, a hand-worked example
(tests/golden/hand_example.json) and an independent nested-loop Python
forward (tests/bruteforce.py).
"""
import json
import os

import numpy as np
import pytest
import torch

import bruteforce
from oracle import rec_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ formats
def test_half_decode_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([orc.half_to_double(int(b)) for b in bits])
    finite = np.isfinite(want)
    assert np.array_equal(got[finite], want[finite])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want))
    assert np.array_equal(np.signbit(got[finite]), np.signbit(want[finite]))


def test_round_bf16_matches_library_rounding():
    g = rng(1)
    xs = np.concatenate([
        g.standard_normal(2000) * 10.0 ** g.integers(-6, 6, 2000),
        # exact ties between neighbouring bf16 values, both parities
        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(2.0 + 2.0 ** -7), 0.0, 1.0, -3.5]),
        np.array([np.float32(1.0 + 2.0 ** -8 + 2.0 ** -20)]),
    ]).astype(np.float32)
    want = torch.from_numpy(xs).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([orc.round_bf16(float(x)) for x in xs])
    assert np.array_equal(got, want)


def test_sigmoid_identities():
    assert orc.sigmoid(0.0) == 0.5
    for x in [0.1, 1.0, 3.7, 12.0]:
        assert abs(orc.sigmoid(-x) - (1.0 - orc.sigmoid(x))) < 1e-15
    assert abs(orc.sigmoid(np.log(3.0)) - 0.75) < 1e-15


# ------------------------------------------------------------------ S0 scan
def test_offsets_identities_and_bruteforce():
    g = rng(2)
    for n in [0, 1, 2, 63, 64, 65, 1000, 5000]:
        lens = g.integers(0, 200, n).astype(np.int32)
        off, rc, _ = orc.offsets(lens)
        assert rc == 0 and off[0] == 0 and off[-1] == lens.sum(dtype=np.int64)
        assert np.array_equal(np.diff(off), lens)
        acc, brute = 0, [0]
        for v in lens:
            acc += int(v)
            brute.append(acc)
        assert off.tolist() == brute


def test_offsets_beyond_int32_and_negative():
    lens = np.full(3000, 1_000_000, dtype=np.int32)       # total 3e9 > 2^31
    off, rc, _ = orc.offsets(lens)
    assert rc == 0 and off[-1] == 3_000_000_000
    lens = np.array([3, 4, -1, 5, -2], dtype=np.int32)
    off, rc, bad = orc.offsets(lens)
    assert rc == -1 and bad == 2


# ------------------------------------------------------------------ S1 pool
def _tables(g, T, R, D, dtype):
    return [(g.uniform(-0.05, 0.05, (R, D))).astype(dtype) for _ in range(T)]


def _bags(g, T, B, R, lo, hi):
    lens = g.integers(lo, hi + 1, T * B).astype(np.int32)
    idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
    return idx, lens


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_pool_single_index_is_the_row(dtype):
    # Pooling factor 1 degenerates to a plain lookup (Sec. V, NMP emulation note).
    g = rng(3)
    T, R, D, B = 3, 50, 8, 7
    tabs = _tables(g, T, R, D, dtype)
    lens = np.ones(T * B, dtype=np.int32)
    idx = g.integers(0, R, T * B).astype(np.int32)
    P, _, nbad, _ = orc.pool(tabs, idx, lens, B)
    assert nbad == 0
    for t in range(T):
        for b in range(B):
            assert np.array_equal(P[b, t], tabs[t][idx[t * B + b]].astype(np.float64))


def test_pool_order_invariance_exact_for_half_tables():
    # fp16 values below 0.05 are multiples of 2^-24 and 200 of them stay below
    # 2^4, so an fp64 sum is exact and cannot depend on the order.
    g = rng(4)
    T, R, D, B = 2, 300, 16, 5
    tabs = _tables(g, T, R, D, np.float16)
    idx, lens = _bags(g, T, B, R, 150, 200)
    P0, _, _, _ = orc.pool(tabs, idx, lens, B)
    off = np.concatenate([[0], np.cumsum(lens)])
    idx2 = idx.copy()
    for k in range(T * B):
        seg = idx2[off[k]:off[k + 1]]
        g.shuffle(seg)
    P1, _, _, _ = orc.pool(tabs, idx2, lens, B)
    assert np.array_equal(P0, P1)
    tabs32 = _tables(g, T, R, D, np.float32)
    Q0, _, _, _ = orc.pool(tabs32, idx, lens, B)
    Q1, _, _, _ = orc.pool(tabs32, idx2, lens, B)
    assert np.allclose(Q0, Q1, rtol=1e-12, atol=1e-15)


def test_pool_closed_forms():
    g = rng(5)
    T, R, D, B = 3, 5000, 4, 9
    idx, lens = _bags(g, T, B, R, 0, 40)
    ones = [np.ones((R, D), dtype=np.float32) for _ in range(T)]
    P, A, nbad, _ = orc.pool(ones, idx, lens, B, want_abs=True)
    assert nbad == 0
    want = lens.reshape(T, B).T.astype(np.float64)          # [B, T]
    assert np.array_equal(P, np.repeat(want[:, :, None], D, axis=2))
    assert np.array_equal(A, P)
    # table whose row r holds (r mod 2048) + column: the pooled value names the ids
    rowid = [((np.arange(R) % 2048)[:, None] + np.arange(D)[None, :]).astype(np.float32)
             for _ in range(T)]
    P, _, _, _ = orc.pool(rowid, idx, lens, B)
    off = np.concatenate([[0], np.cumsum(lens)])
    for t in range(T):
        for b in range(B):
            ids = idx[off[t * B + b]:off[t * B + b + 1]].astype(np.int64)
            for d in range(D):
                assert P[b, t, d] == float((ids % 2048 + d).sum())


def test_pool_duplicates_scaling_and_empty():
    g = rng(6)
    T, R, D, B = 1, 20, 8, 3
    tabs = _tables(g, T, R, D, np.float32)
    lens = np.array([2, 0, 3], dtype=np.int32)
    idx = np.array([7, 7, 1, 2, 1], dtype=np.int32)
    P, _, _, _ = orc.pool(tabs, idx, lens, B)
    r = tabs[0].astype(np.float64)
    assert np.array_equal(P[0, 0], 2.0 * r[7])
    assert np.array_equal(P[1, 0], np.zeros(D))
    assert np.array_equal(P[2, 0], (r[1] + r[2]) + r[1])
    P2, _, _, _ = orc.pool([tabs[0] * np.float32(2)], idx, lens, B)
    assert np.array_equal(P2, 2.0 * P)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_pool_equals_count_matrix_product(dtype):
    g = rng(7)
    T, R, D, B = 4, 37, 8, 6
    tabs = _tables(g, T, R, D, dtype)
    idx, lens = _bags(g, T, B, R, 0, 25)
    P, A, _, _ = orc.pool(tabs, idx, lens, B, want_abs=True)
    off = np.concatenate([[0], np.cumsum(lens)])
    for t in range(T):
        M = np.zeros((B, R))
        for b in range(B):
            np.add.at(M[b], idx[off[t * B + b]:off[t * B + b + 1]], 1.0)
        assert np.allclose(P[:, t, :], M @ tabs[t].astype(np.float64), rtol=1e-13, atol=1e-15)
        assert np.allclose(A[:, t, :], M @ np.abs(tabs[t].astype(np.float64)), rtol=1e-13)


def test_pool_table_major_layout():
    # bag (t, b) is entry t*B + b of lengths; a sample-major reading would
    # swap these two results.
    tabs = [np.array([[1.0], [10.0]], np.float32), np.array([[100.0], [1000.0]], np.float32)]
    B = 2
    lens = np.array([1, 2, 2, 1], dtype=np.int32)        # (t0,b0) (t0,b1) (t1,b0) (t1,b1)
    idx = np.array([0, 1, 1, 0, 1, 0], dtype=np.int32)
    P, _, _, _ = orc.pool(tabs, idx, lens, B)
    assert P[:, :, 0].tolist() == [[1.0, 1100.0], [20.0, 100.0]]


def test_pool_out_of_range_id_contributes_zero_and_is_reported():
    tabs = [np.arange(12, dtype=np.float32).reshape(6, 2)]
    lens = np.array([3, 2], dtype=np.int32)
    idx = np.array([1, 6, 2, -1, 5], dtype=np.int32)
    P, _, nbad, first = orc.pool(tabs, idx, lens, 2)
    assert nbad == 2 and first == 1
    assert P[0, 0].tolist() == [2.0 + 4.0, 3.0 + 5.0]
    assert P[1, 0].tolist() == [10.0, 11.0]


# ------------------------------------------------------------------ S2 / S4
def test_fc_matches_numpy_and_special_cases():
    g = rng(8)
    B, n_in, n_out = 5, 37, 11
    x = g.standard_normal((B, n_in))
    W = g.standard_normal((n_out, n_in)).astype(np.float32)
    b = g.standard_normal(n_out).astype(np.float32)
    lin = x @ W.astype(np.float64).T + b.astype(np.float64)
    assert np.allclose(orc.fc(x, W, b, False), lin, rtol=1e-13, atol=1e-13)
    assert np.allclose(orc.fc(x, W, b, True), np.maximum(lin, 0.0), rtol=1e-13, atol=1e-13)
    assert (orc.fc(x, W, b, True) >= 0).all() and (lin < 0).any()
    # identity weights, zero bias: ReLU(x)
    eye = np.eye(n_in, dtype=np.float32)
    assert np.array_equal(orc.fc(x, eye, np.zeros(n_in, np.float32), True), np.maximum(x, 0.0))
    # zero weights: the bias, exactly
    assert np.array_equal(orc.fc(x, np.zeros_like(W), b, False),
                          np.repeat(b.astype(np.float64)[None, :], B, 0))
    # zero padding of the contraction dimension changes nothing
    xp = np.concatenate([x, np.zeros((B, 5))], axis=1)
    Wp = np.concatenate([W, g.standard_normal((n_out, 5)).astype(np.float32)], axis=1)
    assert np.array_equal(orc.fc(xp, Wp, b, False), orc.fc(x, W, b, False))
    # W is [out, in]: a transposed reading fails on a non-square layer
    W2 = np.zeros((2, 3), np.float32)
    W2[1, 2] = 1.0
    y = orc.fc(np.array([[1.0, 2.0, 3.0]]), W2, np.zeros(2, np.float32), False)
    assert y.tolist() == [[0.0, 3.0]]


def test_fc_bf16_mirror_rounds_inputs_not_accumulation():
    g = rng(9)
    B, n_in, n_out = 4, 64, 8
    x = g.standard_normal((B, n_in))
    W = (g.standard_normal((n_out, n_in)) / 8).astype(np.float32)
    b = g.standard_normal(n_out).astype(np.float32)
    xr = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    Wr = torch.from_numpy(W).to(torch.bfloat16).to(torch.float64).numpy()
    want = xr @ Wr.T + b.astype(np.float64)
    got = orc.fc(x, W, b, False, orc.BF16_MIRROR)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)
    assert not np.allclose(got, orc.fc(x, W, b, False), rtol=1e-6, atol=0)


# ------------------------------------------------------------------ S3
def test_gram_symmetry_norms_and_library_product():
    g = rng(10)
    B, T, D = 3, 6, 8
    x0 = g.standard_normal((B, D))
    P = g.standard_normal((B, T, D))
    Z = orc.gram(x0, P)
    X = np.concatenate([x0[:, None, :], P], axis=1)
    assert np.array_equal(Z, np.transpose(Z, (0, 2, 1)))
    assert np.allclose(np.diagonal(Z, axis1=1, axis2=2), (X * X).sum(-1), rtol=1e-14)
    assert np.allclose(Z, X @ np.transpose(X, (0, 2, 1)), rtol=1e-13, atol=1e-14)


def test_interact_order_width_and_constant_cases():
    g = rng(11)
    B, T, D = 2, 5, 8
    x0 = g.standard_normal((B, D))
    P = g.standard_normal((B, T, D))
    out = orc.interact(x0, P)
    assert out.shape == (B, D + T * (T + 1) // 2)
    X = np.concatenate([x0[:, None, :], P], axis=1)
    G = X @ np.transpose(X, (0, 2, 1))
    for b in range(B):
        assert np.array_equal(out[b, :D], x0[b])                 # dense part first
        want = [G[b, i, j] for i in range(1, T + 1) for j in range(i)]
        assert np.allclose(out[b, D:], want, rtol=1e-13, atol=1e-14)
    # all-ones vectors: every term is D
    out = orc.interact(np.ones((B, D)), np.ones((B, T, D)))
    assert np.array_equal(out[:, D:], np.full((B, T * (T + 1) // 2), float(D)))
    # distinct one-hot vectors: every term is 0
    eye = np.eye(D)
    out = orc.interact(np.tile(eye[0], (B, 1)), np.tile(eye[1:T + 1][None], (B, 1, 1)))
    assert not out[:, D:].any()
    # zero tables: only x0 survives
    out = orc.interact(x0, np.zeros((B, T, D)))
    assert not out[:, D:].any() and np.array_equal(out[:, :D], x0)


# ------------------------------------------------------------------ whole
def _toy(g, T=2, R=5, D=4, B=3, bottom=(3, 4, 4), top_hidden=(3,), dtype=np.float32):
    tabs = [g.uniform(-1, 1, (R, D)).astype(dtype) for _ in range(T)]
    lens = g.integers(0, 4, T * B).astype(np.int32)
    idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
    dense = g.standard_normal((B, bottom[0])).astype(np.float32)
    def stack(widths):
        return [(g.standard_normal((widths[i + 1], widths[i])).astype(np.float32),
                 g.standard_normal(widths[i + 1]).astype(np.float32))
                for i in range(len(widths) - 1)]
    topw = (D + T * (T + 1) // 2,) + tuple(top_hidden) + (1,)
    return dense, tabs, idx, lens, stack(bottom), stack(topw)


@pytest.mark.parametrize("seed,dtype", [(12, np.float32), (13, np.float16), (14, np.float32)])
def test_forward_matches_nested_loop_python(seed, dtype):
    g = rng(seed)
    dense, tabs, idx, lens, bottom, top = _toy(g, dtype=dtype)
    got = orc.forward(dense, tabs, idx, lens, bottom, top)
    want = bruteforce.forward(dense.tolist(), [t.tolist() for t in tabs], idx.tolist(),
                              lens.tolist(), [(W.tolist(), b.tolist()) for W, b in bottom],
                              [(W.tolist(), b.tolist()) for W, b in top])
    for key in ["pooled", "bottom_out", "interact", "logits"]:
        assert np.allclose(got[key], np.array(want[key]), rtol=1e-12, atol=1e-12), key


def test_forward_hand_worked_example():
    with open(os.path.join(GOLDEN, "hand_example.json")) as f:
        ex = json.load(f)
    tabs = [np.array(t, dtype=np.float32) for t in ex["tables"]]
    lens = np.array(ex["lengths_table_major"], dtype=np.int32)
    idx = np.array(ex["indices"], dtype=np.int32)
    dense = np.array(ex["dense"], dtype=np.float32)
    mk = lambda layers: [(np.array(L["W"], np.float32), np.array(L["b"], np.float32)) for L in layers]
    off, rc, _ = orc.offsets(lens)
    assert rc == 0 and off.tolist() == ex["expect"]["offsets"]
    for tabs_v in (tabs, [t.astype(np.float16) for t in tabs]):
        got = orc.forward(dense, tabs_v, idx, lens, mk(ex["bottom"]), mk(ex["top"]))
        for key in ["pooled", "bottom_out", "interact", "logits"]:
            assert np.array_equal(got[key], np.array(ex["expect"][key], dtype=np.float64)), key
    # the same example is exactly representable in bf16, so the mirror mode agrees
    got = orc.forward(dense, tabs, idx, lens, mk(ex["bottom"]), mk(ex["top"]), orc.BF16_MIRROR)
    assert np.array_equal(got["logits"], np.array(ex["expect"]["logits"]))


def test_forward_steps_compose():
    g = rng(15)
    dense, tabs, idx, lens, bottom, top = _toy(g, T=3, R=9, D=4, B=4, bottom=(5, 6, 4), top_hidden=(7, 3))
    got = orc.forward(dense, tabs, idx, lens, bottom, top)
    P, _, _, _ = orc.pool(tabs, idx, lens, 4)
    assert np.array_equal(got["pooled"], P)
    h = dense.astype(np.float64)
    for W, b in bottom:
        h = orc.fc(h, W, b, True)
    assert np.array_equal(got["bottom_out"], h)
    z = orc.interact(h, P)
    assert np.array_equal(got["interact"], z)
    for i, (W, b) in enumerate(top):
        z = orc.fc(z, W, b, i + 1 < len(top))
    assert np.array_equal(got["logits"], z[:, 0])


def test_forward_bf16_mirror_narrows_matrix_layers_only():
    # Mirror mode narrows operands of every layer that is a matrix product; the
    # one-output last layer is a dot product and stays un-narrowed.
    g = rng(19)
    dense, tabs, idx, lens, bottom, top = _toy(g, T=3, R=9, D=4, B=4, bottom=(5, 6, 4), top_hidden=(7, 3))
    got = orc.forward(dense, tabs, idx, lens, bottom, top, orc.BF16_MIRROR)
    P, _, _, _ = orc.pool(tabs, idx, lens, 4)
    h = dense.astype(np.float64)
    for W, b in bottom:
        h = orc.fc(h, W, b, True, orc.BF16_MIRROR)
    z = orc.interact(h, P)
    z = np.vectorize(orc.round_bf16)(z)          # the interaction output is narrowed as well
    assert np.array_equal(got["interact"], z)
    for i, (W, b) in enumerate(top):
        last = i + 1 == len(top)
        z = orc.fc(z, W, b, not last, orc.EXACT if last else orc.BF16_MIRROR)
    assert np.array_equal(got["logits"], z[:, 0])
    assert not np.array_equal(got["logits"], orc.forward(dense, tabs, idx, lens, bottom, top)["logits"])


def test_forward_zero_top_weights_give_last_bias():
    g = rng(16)
    dense, tabs, idx, lens, bottom, top = _toy(g)
    top = [(np.zeros_like(W), b) for W, b in top]
    got = orc.forward(dense, tabs, idx, lens, bottom, top)
    assert np.array_equal(got["logits"], np.full(3, float(top[-1][1][0])))


def test_forward_rejects_bad_width_chain():
    g = rng(17)
    dense, tabs, idx, lens, bottom, top = _toy(g)
    bad_top = [(np.zeros((3, 12), np.float32), np.zeros(3, np.float32)),
               (np.zeros((1, 3), np.float32), np.zeros(1, np.float32))]
    with pytest.raises(ValueError):
        orc.forward(dense, tabs, idx, lens, bottom, bad_top)


def test_threads_do_not_change_results():
    g = rng(18)
    dense, tabs, idx, lens, bottom, top = _toy(g, T=3, R=50, D=8, B=16, bottom=(6, 8), top_hidden=(5,))
    orc.set_threads(1)
    a = orc.forward(dense, tabs, idx, lens, bottom, top)
    orc.set_threads(4)
    b = orc.forward(dense, tabs, idx, lens, bottom, top)
    orc.set_threads(1)
    for key in a:
        assert np.array_equal(a[key], b[key])


# ------------------------------------------------------------------ concatenation model, N towers
def _toy_towers(g, T=3, R=7, D=4, B=4, bottom=(5,), hidden=(6, 3), n_towers=3, dtype=np.float32,
                one_lookup=False):
    tabs = [g.uniform(-1, 1, (R, D)).astype(dtype) for _ in range(T)]
    lens = (np.ones(T * B) if one_lookup else g.integers(0, 4, T * B)).astype(np.int32)
    idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
    dense = g.standard_normal((B, bottom[0])).astype(np.float32)
    def stack(widths):
        return [(g.standard_normal((widths[i + 1], widths[i])).astype(np.float32),
                 g.standard_normal(widths[i + 1]).astype(np.float32))
                for i in range(len(widths) - 1)]
    topw = (bottom[-1] + T * D,) + tuple(hidden) + (1,)
    return dense, tabs, idx, lens, stack(bottom), [stack(topw) for _ in range(n_towers)]


def test_concat_is_numpy_concatenate():
    g = rng(30)
    x0 = g.standard_normal((5, 3))
    P = g.standard_normal((5, 4, 6))
    assert np.array_equal(orc.concat(x0, P), np.concatenate([x0, P.reshape(5, 24)], axis=1))


@pytest.mark.parametrize("seed,dtype,bottom", [(31, np.float32, (5,)), (32, np.float16, (5, 6, 3)),
                                               (33, np.float32, (2, 4))])
def test_towers_forward_matches_nested_loop_python(seed, dtype, bottom):
    g = rng(seed)
    dense, tabs, idx, lens, bot, towers = _toy_towers(g, dtype=dtype, bottom=bottom)
    got = orc.forward_towers(dense, tabs, idx, lens, bot, towers)
    want = bruteforce.forward_towers(dense.tolist(), [t.tolist() for t in tabs], idx.tolist(), lens.tolist(),
                                     [(W.tolist(), b.tolist()) for W, b in bot],
                                     [[(W.tolist(), b.tolist()) for W, b in tw] for tw in towers])
    assert np.allclose(got["concat"], np.array(want["concat"]), rtol=1e-12, atol=1e-12)
    assert np.allclose(got["logits"], np.array(want["logits"]), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_towers_one_lookup_reproduces_rows_bit_for_bit(dtype):
    # One id per bag: no reduction happens, the concatenation holds the stored rows.
    g = rng(34)
    dense, tabs, idx, lens, bot, towers = _toy_towers(g, T=4, R=11, D=8, B=5, dtype=dtype, one_lookup=True)
    got = orc.forward_towers(dense, tabs, idx, lens, bot, towers)
    T, B, D, w0 = 4, 5, 8, 5
    assert np.array_equal(got["concat"][:, :w0], dense.astype(np.float64))   # no Bottom-FC: dense as given
    for t in range(T):
        for b in range(B):
            row = tabs[t][idx[t * B + b]].astype(np.float64)
            assert np.array_equal(got["concat"][b, w0 + t * D:w0 + (t + 1) * D], row)


def test_towers_reduce_to_single_layers_and_are_independent():
    g = rng(35)
    dense, tabs, idx, lens, bot, towers = _toy_towers(g, bottom=(5, 4), n_towers=3)
    got = orc.forward_towers(dense, tabs, idx, lens, bot, towers)
    # every tower is the plain layer chain applied to the same concatenated vector
    z = got["concat"]
    for k, tw in enumerate(towers):
        h = z
        for i, (W, b) in enumerate(tw):
            h = h @ W.astype(np.float64).T + b.astype(np.float64)
            if i + 1 < len(tw):
                h = np.maximum(h, 0.0)
        assert np.allclose(got["logits"][:, k], h[:, 0], rtol=1e-12, atol=1e-12)
    # permuting the towers permutes the columns; a single tower gives its column
    perm = [2, 0, 1]
    got_p = orc.forward_towers(dense, tabs, idx, lens, bot, [towers[k] for k in perm])
    assert np.array_equal(got_p["logits"], got["logits"][:, perm])
    one = orc.forward_towers(dense, tabs, idx, lens, bot, [towers[1]])
    assert np.array_equal(one["logits"][:, 0], got["logits"][:, 1])
    # equal weights, equal logits; zero weights, the last bias
    same = orc.forward_towers(dense, tabs, idx, lens, bot, [towers[0], towers[0]])
    assert np.array_equal(same["logits"][:, 0], same["logits"][:, 1])
    zero = [[(np.zeros_like(W), b) for W, b in tw] for tw in towers]
    zl = orc.forward_towers(dense, tabs, idx, lens, bot, zero)["logits"]
    assert np.array_equal(zl, np.tile([float(tw[-1][1][0]) for tw in zero], (4, 1)))


def test_towers_steps_compose_and_mirror_narrows_matrix_layers_only():
    g = rng(36)
    dense, tabs, idx, lens, bot, towers = _toy_towers(g, bottom=(5, 6), n_towers=2)
    P, _, _, _ = orc.pool(tabs, idx, lens, 4)
    for mode in (orc.EXACT, orc.BF16_MIRROR):
        got = orc.forward_towers(dense, tabs, idx, lens, bot, towers, mode)
        assert np.array_equal(got["pooled"], P)
        h = dense.astype(np.float64)
        for W, b in bot:
            h = orc.fc(h, W, b, True, mode)
        assert np.array_equal(got["bottom_out"], h)
        z = orc.concat(h, P)
        if mode == orc.BF16_MIRROR:
            z = np.vectorize(orc.round_bf16)(z)
        assert np.array_equal(got["concat"], z)
        for k, tw in enumerate(towers):
            y = z
            for i, (W, b) in enumerate(tw):
                last = i + 1 == len(tw)
                y = orc.fc(y, W, b, not last, orc.EXACT if last else mode)
            assert np.array_equal(got["logits"][:, k], y[:, 0])


def test_towers_reject_bad_width_chain():
    g = rng(37)
    dense, tabs, idx, lens, bot, towers = _toy_towers(g)
    bad = [[(np.zeros((3, 9), np.float32), np.zeros(3, np.float32)),
            (np.zeros((1, 3), np.float32), np.zeros(1, np.float32))]]
    with pytest.raises(ValueError):
        orc.forward_towers(dense, tabs, idx, lens, bot, bad)


def test_bf16_mirror_per_sample_spread_against_exact_mode():
    """What bf16 operands alone (no device) do to a logit: on a whole rmc1-style
    batch the mirror stays within 2e-2 of the exact mode batch-wise, its median
    per-sample deviation is a few 1e-3 of max(|o|, rms), and at most a sample or
    two in a thousand cross 2e-2.  This is the spread the device is allowed."""
    from paper_2203_07424_amd import synth
    w = synth.WORKLOADS["rmc1"]
    bottom, top = synth.draw_mlp(w, "bottom"), synth.draw_mlp(w, "top")
    batch = synth.draw_batch(w, 0)
    tabs, cidx = synth.compact_tables(w, batch, w.batch)
    exact = orc.forward(batch.dense, tabs, cidx, batch.lengths, bottom, top)["logits"]
    mirror = orc.forward(batch.dense, tabs, cidx, batch.lengths, bottom, top, orc.BF16_MIRROR)["logits"]
    assert np.linalg.norm(mirror - exact) <= 2e-2 * np.linalg.norm(exact)
    rms = np.sqrt((exact ** 2).mean())
    ratio = np.abs(mirror - exact) / np.maximum(np.abs(exact), rms)
    assert 5e-4 < np.median(ratio) < 1e-2
    assert ratio.max() < 4e-2 and (ratio > 2e-2).sum() <= 3
