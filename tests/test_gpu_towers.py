"""Parity of the concatenation model with N Predict-FC towers (Table I, row
MT-WnD: one lookup per table, no pooling, no Bottom-FC) against the CPU oracle,
through the C boundary.

The Predict-FC input is bf16 on the device: with one id per bag it must hold the
stored rows narrowed once (bit-exact against the oracle's bf16 mirror); with
longer bags it is the fp32 sum narrowed, compared within one bf16 rounding.
Logits: 2e-2 relative per tower against the exact oracle, 5e-3 per sample
against the mirror.
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


def stacks(g, F, hidden_b, T, D, hidden_t, n_towers):
    def stack(ws):
        return [((g.standard_normal((ws[i + 1], ws[i])) * ws[i] ** -0.5).astype(np.float32),
                 (g.standard_normal(ws[i + 1]) * ws[i] ** -0.5).astype(np.float32))
                for i in range(len(ws) - 1)]
    bw = (F,) + tuple(hidden_b)
    width = bw[-1] + T * D
    return stack(bw), [stack((width,) + tuple(hidden_t) + (1,)) for _ in range(n_towers)]


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Bit patterns of values that are exactly representable in bf16."""
    return (x.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)


CASES = [
    # T, R, D, dtype, B, F, hidden_b, hidden_t, towers, (lo, hi) ids per bag
    (5, 400, 32, np.float32, 70, 24, (40,), (96, 72), 3, (1, 1)),     # one lookup, ragged widths
    (26, 300, 64, np.float16, 130, 64, (), (256, 128, 64), 4, (1, 1)),  # the MT-WnD shape, fused last dot
    (4, 200, 16, np.float16, 33, 13, (), (48,), 2, (1, 1)),           # dense part not 16-byte aligned
    (3, 500, 32, np.float32, 65, 7, (20, 12), (64,), 8, (0, 3)),      # short ragged bags, 8 towers
    (6, 250, 64, np.float16, 40, 16, (), (130, 70), 2, (0, 60)),      # long bags: one wave per bag
    (2, 100, 8, np.float32, 257, 5, (), (), 5, (1, 1)),               # towers of one (one-output) layer
    (3, 100, 256, np.float32, 19, 8, (16,), (32,), 1, (1, 2)),        # 1 KB rows, one tower
    (3, 100, 32, np.float16, 90, 8, (), (40, 300), 3, (1, 1)),        # last hidden layer too wide to fuse the dot
    (3, 100, 32, np.float16, 300, 8, (), (40, 200), 2, (1, 1)),       # dot fused into a 256-wide last hidden layer
]


@pytest.mark.parametrize("T,R,D,dtype,B,F,hb,ht,nt,lohi", CASES)
def test_concat_towers_against_oracle(binding, T, R, D, dtype, B, F, hb, ht, nt, lohi):
    say("towers case", T, R, D, dtype.__name__, B, F, hb, ht, nt, lohi)
    g = np.random.default_rng(500 + T + B)
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(dtype) for _ in range(T)]
    lens = g.integers(lohi[0], lohi[1] + 1, T * B).astype(np.int32)
    idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
    bottom, towers = stacks(g, F, hb, T, D, ht, nt)
    dense = g.standard_normal((B, F)).astype(np.float32)
    m = H.make_model(binding, tabs, bottom, towers, B + 5, max(idx.size, 1), F, interaction="concat")
    logits = H.run(m, synth.Batch(dense, idx, lens))
    assert m.check() == (binding.REC_OK, -1)
    assert logits.shape == ((B,) if nt == 1 else (B, nt))
    exact = orc.forward_towers(dense, tabs, idx, lens, bottom, towers, orc.EXACT)
    mirror = orc.forward_towers(dense, tabs, idx, lens, bottom, towers, orc.BF16_MIRROR)
    off, _, _ = orc.offsets(lens)
    assert np.array_equal(m.debug_offsets().cpu().numpy().astype(np.int64), off)

    # Predict-FC input
    w0 = (F,) + tuple(hb)
    w0 = w0[-1]
    width = w0 + T * D
    z_t = m.debug_interact()
    z = z_t.float().cpu().numpy().astype(np.float64)
    assert not z[:, width:].any()
    emb, emb_m = z[:, w0:width], mirror["concat"][:, w0:]
    if lohi == (1, 1):
        assert np.array_equal(bf16_bits(emb), bf16_bits(emb_m))     # rows narrowed once: bit-exact
    else:
        scale = np.abs(exact["concat"][:, w0:])
        assert (np.abs(emb - exact["concat"][:, w0:]) <= 2.0 ** -8 * scale + 1e-6).all()
    if not hb:
        assert np.array_equal(bf16_bits(z[:, :w0]), bf16_bits(mirror["concat"][:, :w0]))  # dense as given
    else:
        s = np.abs(mirror["bottom_out"]).max() + 1e-30
        assert np.abs(z[:, :w0] - mirror["concat"][:, :w0]).max() <= 2.0 ** -7 * s
        x0 = m.debug_bottom_out().cpu().numpy().astype(np.float64)
        assert np.abs(x0 - mirror["bottom_out"]).max() <= 2e-3 * s
    # with no Bottom-FC / in this model the fp32 buffers are not produced
    assert binding.rec_debug_get(m.handle, binding.REC_DBG_POOLED)[0] == binding.REC_ERR_STATE
    if not hb:
        assert binding.rec_debug_get(m.handle, binding.REC_DBG_BOTTOM_OUT)[0] == binding.REC_ERR_STATE

    want_e = exact["logits"][:, 0] if nt == 1 else exact["logits"]
    want_m = mirror["logits"][:, 0] if nt == 1 else mirror["logits"]
    H.check_logits(logits, want_e, want_m)
    m.close()


def test_short_bags_in_the_interaction_model(binding):
    # Bags of a few ids share a wavefront in either model; here the fp32 pooled
    # sums of the pairwise-dot model are checked to 1e-5.
    say("short bags, dot model")
    g = np.random.default_rng(77)
    for (T, R, D, dtype, B, hi) in [(3, 900, 32, np.float32, 1111, 3), (2, 700, 64, np.float16, 515, 4),
                                    (4, 300, 8, np.float16, 300, 2), (1, 50, 128, np.float32, 70, 1)]:
        tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(dtype) for _ in range(T)]
        lens = g.integers(0, hi + 1, T * B).astype(np.int32)
        idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
        bw = [((g.standard_normal((D, 4)) * 0.5).astype(np.float32), np.zeros(D, np.float32))]
        tw = [((g.standard_normal((1, D + T * (T + 1) // 2)) * 0.1).astype(np.float32), np.zeros(1, np.float32))]
        dense = g.standard_normal((B, 4)).astype(np.float32)
        m = H.make_model(binding, tabs, bw, tw, B, max(idx.size, 1), 4)
        H.run(m, synth.Batch(dense, idx, lens))
        assert m.check() == (binding.REC_OK, -1)
        P, A, nbad, _ = orc.pool(tabs, idx, lens, B, want_abs=True)
        assert nbad == 0
        H.check_pooled(m.debug_pooled().cpu().numpy(), P, A)
        m.close()


def test_short_bags_report_ids_outside_the_table(binding):
    say("short bags, bad ids")
    g = np.random.default_rng(78)
    T, R, D, B = 3, 60, 32, 20
    tabs = [g.uniform(-1, 1, (R, D)).astype(np.float32) for _ in range(T)]
    bottom, towers = stacks(g, 6, (), T, D, (16,), 2)
    lens = np.ones(T * B, dtype=np.int32)
    idx = g.integers(0, R, T * B).astype(np.int32)
    idx[17] = R + 5
    idx[41] = -1
    dense = g.standard_normal((B, 6)).astype(np.float32)
    m = H.make_model(binding, tabs, bottom, towers, B, idx.size, 6, interaction="concat")
    logits = H.run(m, synth.Batch(dense, idx, lens))
    assert m.check() == (binding.REC_ERR_INDEX_RANGE, 17)
    mirror = orc.forward_towers(dense, tabs, idx, lens, bottom, towers, orc.BF16_MIRROR)   # bad ids add zero
    z = m.debug_interact().float().cpu().numpy().astype(np.float64)
    assert np.array_equal(bf16_bits(z[:, 6:6 + T * D]), bf16_bits(mirror["concat"][:, 6:]))
    assert not z[17 % B, 6 + (17 // B) * D:6 + (17 // B + 1) * D].any()
    H.check_logits(logits, mirror["logits"], None)
    m.close()


def test_dot_model_without_bottom_fc_and_with_towers(binding):
    # The two extensions are independent of the model shape: pairwise dots with
    # the dense features used as they are, several towers on the interaction.
    say("dot model, no Bottom-FC, towers")
    g = np.random.default_rng(79)
    T, R, D, B = 4, 200, 32, 50
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(np.float16) for _ in range(T)]
    lens = g.integers(0, 30, T * B).astype(np.int32)
    idx = g.integers(0, R, int(lens.sum())).astype(np.int32)
    dense = (g.standard_normal((B, D)) * 0.1).astype(np.float32)
    width = D + T * (T + 1) // 2
    def stack(ws):
        return [((g.standard_normal((ws[i + 1], ws[i])) * ws[i] ** -0.5).astype(np.float32),
                 (g.standard_normal(ws[i + 1]) * ws[i] ** -0.5).astype(np.float32))
                for i in range(len(ws) - 1)]
    towers = [stack((width, 48, 1)) for _ in range(3)]
    m = H.make_model(binding, tabs, [], towers, B, idx.size, D)
    logits = H.run(m, synth.Batch(dense, idx, lens))
    assert m.check() == (binding.REC_OK, -1)
    for k in range(3):
        exact = orc.forward(dense, tabs, idx, lens, [], towers[k], orc.EXACT)
        mirror = orc.forward(dense, tabs, idx, lens, [], towers[k], orc.BF16_MIRROR)
        H.check_logits(logits[:, k], exact["logits"], mirror["logits"])
    m.close()


def test_tiny_tower_workload_full_batch(binding):
    w = synth.WORKLOADS["mtwnd-tiny"]
    say("workload", w.name)
    m, bottom, towers = H.make_workload_model(binding, w)
    batch = synth.draw_batch(w, 0)
    logits = H.run(m, batch)
    assert m.check() == (binding.REC_OK, -1)
    tabs = [synth.full_table(w, t) for t in range(w.num_tables)]
    exact = orc.forward_towers(batch.dense, tabs, batch.indices, batch.lengths, bottom, towers, orc.EXACT)
    mirror = orc.forward_towers(batch.dense, tabs, batch.indices, batch.lengths, bottom, towers, orc.BF16_MIRROR)
    H.check_logits(logits, exact["logits"], mirror["logits"])
    m.close()


def test_full_size_tower_workload_sampled_against_oracle(binding):
    w = synth.WORKLOADS["mtwnd"]
    say("workload", w.name, "batch", w.batch)
    m, bottom, towers = H.make_workload_model(binding, w)
    cdf = synth.zipf_cdf(w.rows, float(w.index_dist[1]))
    batch = synth.draw_batch(w, 1, cdf)
    logits = H.run(m, batch)
    assert m.check() == (binding.REC_OK, -1)
    z = m.debug_interact().float().cpu().numpy().astype(np.float64)
    pick = np.random.default_rng(5).choice(w.batch, 48, replace=False)
    pick[:3] = [0, w.batch - 1, w.batch // 2]
    exact = H.oracle_on_slice(w, batch, pick, bottom, towers, orc.EXACT)
    mirror = H.oracle_on_slice(w, batch, pick, bottom, towers, orc.BF16_MIRROR)
    assert np.array_equal(bf16_bits(z[pick, :w.top[0]]), bf16_bits(mirror["concat"]))
    H.check_logits(logits[pick], exact["logits"], mirror["logits"])
    # properties that hold for every sample: finite, and towers differ
    assert np.isfinite(logits).all() and logits.shape == (w.batch, w.towers)
    assert np.abs(logits[:, 0] - logits[:, 1]).max() > 0
    m.close()


@pytest.mark.parametrize("hidden,towers,B", [((1280, 64), 8, 1100), ((640, 200), 8, 1100), ((1024, 512), 2, 2048)])
def test_wide_tower_layers_on_ragged_batches(binding, hidden, towers, B):
    # Layers wide enough, on batches large enough, for the 256-row block tiles
    # (256 x 256 and 256 x 128), with a batch that is not a multiple of the tile.
    say("wide towers", hidden, towers, B)
    g = np.random.default_rng(91)
    T, R, D, F = 6, 300, 32, 8
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(np.float16) for _ in range(T)]
    lens = np.ones(T * B, dtype=np.int32)
    idx = g.integers(0, R, T * B).astype(np.int32)
    bottom, tw = stacks(g, F, (), T, D, hidden, towers)
    dense = g.standard_normal((B, F)).astype(np.float32)
    m = H.make_model(binding, tabs, bottom, tw, B, idx.size, F, interaction="concat")
    logits = H.run(m, synth.Batch(dense, idx, lens))
    assert m.check() == (binding.REC_OK, -1)
    exact = orc.forward_towers(dense, tabs, idx, lens, bottom, tw, orc.EXACT)
    mirror = orc.forward_towers(dense, tabs, idx, lens, bottom, tw, orc.BF16_MIRROR)
    H.check_logits(logits, exact["logits"], mirror["logits"])
    m.close()


def test_tower_model_graph_replay_overlap_and_repeatability(binding):
    """The tower model under a HIP graph (large batch, so the wide-tile kernels
    and their more-than-64-KB LDS grant are inside the capture), with the
    Bottom-FC on the side stream, and run twice: all must give the same bits."""
    say("towers: graph, overlap, repeatability")
    g = np.random.default_rng(93)
    T, R, D, B, F = 6, 300, 32, 1100, 16
    tabs = [g.uniform(-0.05, 0.05, (R, D)).astype(np.float16) for _ in range(T)]
    bottom, towers = stacks(g, F, (48, 24), T, D, (1280, 64), 8)
    m = H.make_model(binding, tabs, bottom, towers, B, T * B, F, interaction="concat")

    def draw():
        return synth.Batch(g.standard_normal((B, F)).astype(np.float32),
                           g.integers(0, R, T * B).astype(np.int32), np.ones(T * B, np.int32))
    first = draw()
    eager0 = H.run(m, first)
    assert np.array_equal(eager0, H.run(m, first))                    # run to run
    m.set_option(binding.REC_OPT_OVERLAP_DENSE, 1)
    assert np.array_equal(eager0, H.run(m, first))                    # side stream
    m.set_option(binding.REC_OPT_OVERLAP_DENSE, 0)
    bufs = (torch.from_numpy(first.dense).cuda(), torch.from_numpy(first.indices).cuda(),
            torch.from_numpy(first.lengths).cuda())
    out = torch.empty((B, 8), dtype=torch.float32, device="cuda")
    cap = binding.CapturedForward(m, [bufs], [out])
    scratch = torch.zeros(1 << 20, device="cuda")
    for rep in range(4):
        b = first if rep == 0 else draw()
        bufs[0].copy_(torch.from_numpy(b.dense))
        bufs[1].copy_(torch.from_numpy(b.indices))
        out.zero_()
        cap.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy().copy()
        scratch.add_(1.0)
        assert np.array_equal(got, H.run(m, b)), rep
        assert m.check() == (binding.REC_OK, -1)
    exact = orc.forward_towers(b.dense, tabs, b.indices, b.lengths, bottom, towers)
    mirror = orc.forward_towers(b.dense, tabs, b.indices, b.lengths, bottom, towers, orc.BF16_MIRROR)
    H.check_logits(got, exact["logits"], mirror["logits"])
    m.close()


@pytest.mark.parametrize("interaction", ["dot", "concat"])
def test_batch_without_any_id(binding, interaction):
    # Every bag empty: nnz = 0 and no index buffer at all.  The embeddings'
    # share of the Predict-FC input is zero, the logits depend on the dense part only.
    say("no ids", interaction)
    g = np.random.default_rng(95)
    T, R, D, B, F = 3, 50, 32, 70, 32
    tabs = [g.uniform(-1, 1, (R, D)).astype(np.float32) for _ in range(T)]
    lens = np.zeros(T * B, dtype=np.int32)
    idx = np.zeros(0, dtype=np.int32)
    dense = g.standard_normal((B, F)).astype(np.float32)
    if interaction == "concat":
        bottom, top = stacks(g, F, (), T, D, (48,), 2)
        oracle = lambda mode: orc.forward_towers(dense, tabs, idx, lens, bottom, top, mode)
    else:
        bottom = []
        width = D + T * (T + 1) // 2
        top = [((g.standard_normal((40, width)) * width ** -0.5).astype(np.float32), np.zeros(40, np.float32)),
               ((g.standard_normal((1, 40)) * 40 ** -0.5).astype(np.float32), np.ones(1, np.float32))]
        oracle = lambda mode: orc.forward(dense, tabs, idx, lens, bottom, top, mode)
    m = H.make_model(binding, tabs, bottom, top, B, 16, F, interaction=interaction)
    d = torch.from_numpy(dense).cuda()
    l = torch.from_numpy(lens).cuda()
    out = torch.empty((B, 2) if interaction == "concat" else (B,), dtype=torch.float32, device="cuda")
    assert binding.rec_forward(m.handle, d, None, l, B, 0, out) == binding.REC_OK
    torch.cuda.synchronize()
    m.last_batch = B
    assert m.check() == (binding.REC_OK, -1)
    assert not m.debug_offsets().cpu().numpy().any()
    z = m.debug_interact().float().cpu().numpy()
    w0 = F if interaction == "concat" else D
    assert not z[:, w0:].any()                      # embeddings and every dot with them: zero
    got = out.cpu().numpy()
    exact, mirror = oracle(orc.EXACT), oracle(orc.BF16_MIRROR)
    H.check_logits(got, exact["logits"], mirror["logits"])
    m.close()
