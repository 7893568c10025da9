"""The sparse-dense pipeline (REC_OPT_PIPELINE): scan and Bottom-FC on the
caller's stream, pooling launches on two streams in turn, interaction and
Predict-FC on a fourth, four batches in flight.  Same kernels as the in-order
pass, so the logits must be bit-equal to it, and they are held to the oracle's
bars as well.
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


def dev(batch):
    return (torch.from_numpy(batch.dense).cuda(), torch.from_numpy(batch.indices).cuda(),
            torch.from_numpy(batch.lengths).cuda())


@pytest.mark.parametrize("name,own_streams", [("tiny", True), ("tiny", False), ("mtwnd-tiny", True)])
def test_pipelined_forwards_equal_in_order_forwards(binding, name, own_streams):
    """Eleven back-to-back forwards of varying batch size (every frame of the
    workspace is reused at least once), no host synchronisation in between,
    results read after rec_drain(): bit-equal to the in-order model and within
    the bars against the oracle."""
    w = synth.WORKLOADS[name]
    say("pipeline vs in-order", name, own_streams)
    sizes = [w.batch, 37, w.batch, 1, 129, w.batch, 64, 3, w.batch, 200, 5]
    ref, bottom, top = H.make_workload_model(binding, w)
    main = torch.cuda.Stream()
    side = torch.cuda.Stream() if own_streams else None
    pools = (torch.cuda.Stream(), torch.cuda.Stream()) if own_streams else (None, None)
    pm, _, _ = H.make_workload_model(binding, w, share_tables=ref, pipeline=True, dense_stream=side,
                                     pool_streams=pools)
    # Left to itself a pipelined model runs every layer as a kernel of its own (the
    # chain kernel's 8-wave blocks find no room beside pooling), which sums in a
    # different order than a chain: compare like with like.
    ref.set_option(binding.REC_OPT_FUSE_MLP, 0)
    pm.set_option(binding.REC_OPT_FUSE_MLP, 0)
    tabs = [synth.full_table(w, t) for t in range(w.num_tables)]
    batches = [synth.draw_batch(w.with_batch(B), 60 + i) for i, B in enumerate(sizes)]
    data = [dev(b) for b in batches]
    shape = lambda B: (B,) if w.towers == 1 else (B, w.towers)
    want = []
    for b, d in zip(batches, data):
        want.append(ref.forward(*d).cpu().numpy())
    torch.cuda.synchronize()
    outs = [torch.full(shape(B), float("nan"), dtype=torch.float32, device="cuda") for B in sizes]
    with torch.cuda.stream(main):
        for d, o in zip(data, outs):
            pm.forward(*d, o)
        pm.drain()
        got = [o.cpu() for o in outs]          # ordered on `main` behind the drain
    main.synchronize()
    assert pm.check() == (binding.REC_OK, -1) and ref.check() == (binding.REC_OK, -1)
    for i, (g, wnt) in enumerate(zip(got, want)):
        assert np.array_equal(g.numpy(), wnt), i
    for i in (0, 1, 3, 8, 10):
        b = batches[i]
        fwd = orc.forward_towers if w.interaction == "concat" else orc.forward
        exact = fwd(b.dense, tabs, b.indices, b.lengths, bottom, top)
        mirror = fwd(b.dense, tabs, b.indices, b.lengths, bottom, top, orc.BF16_MIRROR)
        H.check_logits(got[i].numpy(), exact["logits"], mirror["logits"])
    # the buffers of the last call's frame can be inspected once it is done
    last = batches[-1]
    assert np.array_equal(np.diff(pm.debug_offsets().cpu().numpy().astype(np.int64)), last.lengths)
    pm.close()
    ref.close()


def test_pipelined_results_are_ordered_behind_drain(binding):
    """Work enqueued on the caller's stream behind rec_drain() sees the logits of
    every call so far, also when drains and forwards alternate, with the
    library's own streams and with ones the caller brings; and every input is
    read in stream order: the uploads sit on the caller's stream behind a long
    kernel, the forwards are enqueued while nothing has arrived yet."""
    w = synth.WORKLOADS["tiny"]
    say("pipeline: ordering behind drain")
    ref, _, _ = H.make_workload_model(binding, w)
    ref.set_option(binding.REC_OPT_FUSE_MLP, 0)
    batches = [synth.draw_batch(w, 80 + i) for i in range(6)]
    data = [dev(b) for b in batches]
    want = [ref.forward(*d).cpu().numpy() for d in data]
    torch.cuda.synchronize()
    pinned = [[torch.from_numpy(a).pin_memory() for a in (b.dense, b.indices, b.lengths)] for b in batches]
    for mode, side, pools in ((1, torch.cuda.Stream(), (torch.cuda.Stream(), torch.cuda.Stream())),
                              (2, None, (None, None))):
        pm, _, _ = H.make_workload_model(binding, w, share_tables=ref, pipeline=True, dense_stream=side,
                                         pool_streams=pools)
        main = torch.cuda.Stream()
        outs = [torch.empty(w.batch, dtype=torch.float32, device="cuda") for _ in data]
        snaps = {}
        # device buffers that hold garbage until the copies on `main` have run
        late = [[torch.full(t.shape, -7, dtype=t.dtype, device="cuda") for t in p] for p in pinned]
        torch.cuda.synchronize()
        with torch.cuda.stream(main):
            torch.cuda._sleep(20_000_000)               # a few milliseconds in front of the uploads
            for p, dv in zip(pinned, late):
                for src, dst in zip(p, dv):
                    dst.copy_(src, non_blocking=True)
            for i, (d, o) in enumerate(zip(late, outs)):
                pm.forward(*d, o)
                if i in (0, 3):                        # a drain in the middle of the run
                    pm.drain()
                    snaps[i] = [outs[j].clone() for j in range(i + 1)]
            pm.drain()
            final = [o.clone() for o in outs]
        main.synchronize()
        for i, sn in snaps.items():
            for j, t in enumerate(sn):
                assert np.array_equal(t.cpu().numpy(), want[j]), (mode, i, j)
        for j, t in enumerate(final):
            assert np.array_equal(t.cpu().numpy(), want[j]), (mode, j)
        assert pm.check() == (binding.REC_OK, -1)
        # the option decides the workspace size: not changeable once one is bound
        assert binding.rec_set_option(pm.handle, binding.REC_OPT_PIPELINE, 0) == binding.REC_ERR_STATE
        pm.close()
    ref.close()


def test_pipelined_stage_timing(binding):
    """Stage events of a pipelined forward: every stage positive."""
    w = synth.WORKLOADS["tiny"]
    say("pipeline: stage events")
    pm, _, _ = H.make_workload_model(binding, w, pipeline=True)
    d = dev(synth.draw_batch(w, 5))
    pm.set_profiling(3, 1)
    for _ in range(3):
        pm.forward(*d)
    pm.drain()
    torch.cuda.synchronize()
    for slot in range(3):
        ms = pm.stage_ms(slot)
        assert all(v > 0 for v in ms.values()), ms
    pm.set_profiling(0)
    pm.close()


def test_pipelined_forwards_in_a_graph(binding):
    """Three pipelined forwards and the drain recorded into one HIP graph (the other
    streams fork from and join the captured one through the library's events);
    every replay, with eager work in between, gives the in-order bits."""
    w = synth.WORKLOADS["tiny"]
    say("pipeline: graph replay")
    ref, _, _ = H.make_workload_model(binding, w)
    ref.set_option(binding.REC_OPT_FUSE_MLP, 0)
    pm, _, _ = H.make_workload_model(binding, w, share_tables=ref, pipeline=True)
    batches = [synth.draw_batch(w, 90 + i) for i in range(3)]
    data = [dev(b) for b in batches]
    want = [ref.forward(*d).cpu().numpy() for d in data]
    outs = [torch.empty(w.batch, dtype=torch.float32, device="cuda") for _ in data]
    torch.cuda.synchronize()
    cap = binding.CapturedForward(pm, data, outs)
    for rep in range(3):
        for o in outs:
            o.zero_()
        cap.replay()
        torch.cuda.synchronize()
        for j, o in enumerate(outs):
            assert np.array_equal(o.cpu().numpy(), want[j]), (rep, j)
        assert np.array_equal(ref.forward(*data[rep]).cpu().numpy(), want[rep])   # eager work between replays
    assert pm.check() == (binding.REC_OK, -1)
    pm.close()
    ref.close()


def test_pipelined_edge_calls(binding):
    """Empty batches, hot-row lists and option changes in a pipelined model."""
    w = synth.WORKLOADS["tiny"].with_batch(96)
    say("pipeline: edge calls")
    ref, _, _ = H.make_workload_model(binding, w)
    ref.set_option(binding.REC_OPT_FUSE_MLP, 0)
    pm, _, _ = H.make_workload_model(binding, w, share_tables=ref, pipeline=True)
    b = synth.draw_batch(w, 11)
    d, i, l = dev(b)
    want = ref.forward(d, i, l).cpu().numpy()
    out = torch.empty(w.batch, dtype=torch.float32, device="cuda")
    pm.forward(d, i, l, out)
    # a batch of zero samples enqueues nothing and leaves the outstanding call alone
    assert binding.rec_forward(pm.handle, d, i, l, 0, 0, out) == binding.REC_OK
    # streams cannot be swapped while work is outstanding on them
    assert binding.rec_set_dense_stream(pm.handle, None) == binding.REC_ERR_STATE
    assert binding.rec_set_pool_streams(pm.handle, None, None) == binding.REC_ERR_STATE
    pm.drain()
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)
    side = torch.cuda.Stream()
    assert binding.rec_set_dense_stream(pm.handle, side) == binding.REC_OK
    pm.dense_stream = side
    pool_a = torch.cuda.Stream()
    assert binding.rec_set_pool_streams(pm.handle, pool_a, None) == binding.REC_OK
    pm.pool_streams = (pool_a, None)
    # hot-row lists: the LDS-cached pooling kernel inside the pipeline, same sums
    hot = synth.profile_hot_rows(w, [3, 4], 64)
    for t in range(w.num_tables):
        pm.load_hot_rows(t, hot[t])
    out2 = torch.empty_like(out)
    pm.forward(d, i, l, out2)
    pm.drain()
    torch.cuda.synchronize()
    exact = orc.forward(b.dense, [synth.full_table(w, t) for t in range(w.num_tables)], b.indices, b.lengths,
                        synth.draw_mlp(w, "bottom"), synth.draw_mlp(w, "top"))
    H.check_logits(out2.cpu().numpy(), exact["logits"])
    assert np.abs(out2.cpu().numpy() - want).max() <= 1e-4 * np.abs(want).max()
    assert pm.check() == (binding.REC_OK, -1)
    pm.close()
    ref.close()


def test_pipelined_faults_are_reported(binding):
    w = synth.WORKLOADS["tiny"].with_batch(64)
    say("pipeline: device faults")
    pm, _, _ = H.make_workload_model(binding, w, pipeline=True)
    b = synth.draw_batch(w, 1)
    bad = b.indices.copy()
    bad[777] = -5
    for idx, expect in ((bad, (binding.REC_ERR_INDEX_RANGE, 777)), (b.indices, (binding.REC_OK, -1))):
        d, i, l = dev(synth.Batch(b.dense, idx, b.lengths))
        out = pm.forward(d, i, l)
        assert pm.check() == expect
        assert torch.isfinite(out).all()
    pm.close()


def test_full_size_pipelined_whole_batches_against_oracle(binding):
    """rmc2 at full size through the pipeline on four streams, twelve batches back
    to back (the benchmark's launch configuration): every sample of the first
    and the last batch against the oracle, all bit-equal to in-order forwards."""
    w = synth.WORKLOADS["rmc2"]
    say("full-size pipelined", w.name)
    ref, bottom, top = H.make_workload_model(binding, w)
    ref.set_option(binding.REC_OPT_FUSE_MLP, 0)
    main, side, pool_a, pool_b = (torch.cuda.Stream() for _ in range(4))
    pm, _, _ = H.make_workload_model(binding, w, share_tables=ref, pipeline=True, dense_stream=side,
                                     pool_streams=(pool_a, pool_b))
    batches = [synth.draw_batch(w, 20 + i) for i in range(4)]
    data = [dev(b) for b in batches]
    want = [ref.forward(*d).cpu().numpy() for d in data]
    outs = [torch.empty(w.batch, dtype=torch.float32, device="cuda") for _ in data]
    torch.cuda.synchronize()
    with torch.cuda.stream(main):
        for rep in range(3):
            for d, o in zip(data, outs):
                pm.forward(*d, o)
        pm.drain()
    main.synchronize()
    assert pm.check() == (binding.REC_OK, -1)
    for i in range(4):
        assert np.array_equal(outs[i].cpu().numpy(), want[i]), i
    for i in (0, 3):
        exact, mirror, P, A = H.oracle_on_batch(w, batches[i], bottom, top)
        H.check_logits(want[i], exact["logits"], mirror["logits"], mirror_rtol=1e-2)   # whole 4096-batch
        if i == 3:      # the last call's frame
            H.check_pooled(pm.debug_pooled().cpu().numpy(), P, A)
    pm.close()
    ref.close()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["rmc1", "rmc3", "mtwnd"])
def test_full_size_pipelined_other_workloads_equal_in_order(binding, name):
    """The other workloads at full size through the pipeline, as the benchmark's
    short legs run them (row loads streaming where the ids are uniform, wide
    layers beside pooling): six batches back to back, bit-equal to in-order
    forwards, which the parity tests hold to the oracle."""
    w = synth.WORKLOADS[name]
    say("full-size pipelined", w.name)
    ref, _, _ = H.make_workload_model(binding, w)
    streams = [torch.cuda.Stream() for _ in range(4)]
    pm, _, _ = H.make_workload_model(binding, w, share_tables=ref, pipeline=True, dense_stream=streams[3],
                                     pool_streams=(streams[1], streams[2]))
    for mm in (ref, pm):
        mm.set_option(binding.REC_OPT_FUSE_MLP, 0)
        mm.set_option(binding.REC_OPT_STREAM_ROWS, int(w.index_dist[0] == "uniform"))
    batches = [synth.draw_batch(w, 40 + i) for i in range(3)]
    data = [dev(b) for b in batches]
    shape = (w.batch,) if w.towers == 1 else (w.batch, w.towers)
    want = [ref.forward(*d).cpu().numpy() for d in data]
    outs = [torch.full(shape, float("nan"), dtype=torch.float32, device="cuda") for _ in range(6)]
    torch.cuda.synchronize()
    with torch.cuda.stream(streams[0]):
        for i, o in enumerate(outs):
            pm.forward(*data[i % 3], o)
        pm.drain()
    streams[0].synchronize()
    assert pm.check() == (binding.REC_OK, -1) and ref.check() == (binding.REC_OK, -1)
    for i, o in enumerate(outs):
        assert np.array_equal(o.cpu().numpy(), want[i % 3]), i
    pm.close()
    ref.close()
    torch.cuda.empty_cache()
