"""rec_forward_static(): the forward pass for callers that cannot allocate.

Called through the C boundary and compared with rec_forward() on the same
inputs: same kernels in the same order, so the logits must be bit-equal; the
oracle check (the bar of the other parity tests) is applied too.  Two calls in
a row, the second on a smaller batch, because the static array keeps what the
first call left behind.
"""
import ctypes as C

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


def _raw_static(b):
    lib = C.CDLL(b.LIB_PATH)
    f = lib.rec_forward_static
    f.restype = C.c_int
    f.argtypes = [C.c_void_p] * 4 + [C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
    return f


def _dev(batch):
    return (torch.from_numpy(batch.dense).cuda(), torch.from_numpy(batch.indices).cuda(),
            torch.from_numpy(batch.lengths).cuda())


@pytest.mark.parametrize("name,b1,b2", [("tiny", 256, 77), ("mtwnd-tiny", 200, 33)])
def test_static_scratch_forward_equals_workspace_forward(binding, name, b1, b2):
    print("static forward", name, b1, b2, flush=True)
    static = _raw_static(binding)
    w = synth.WORKLOADS[name]
    m, bottom, top = H.make_workload_model(binding, w, max_batch=max(b1, b2))
    tabs = [synth.full_table(w, t) for t in range(w.num_tables)]
    stream = torch.cuda.current_stream().cuda_stream
    fault = torch.full((2,), 99, dtype=torch.int64, device="cuda")
    for call, B in enumerate((b1, b2)):
        wb = w.with_batch(B)
        batch = synth.draw_batch(wb, 40 + call)
        d, i, l = _dev(batch)
        shape = (B,) if w.towers == 1 else (B, w.towers)
        want = torch.empty(shape, dtype=torch.float32, device="cuda")
        m.forward(d, i, l, want)
        torch.cuda.synchronize()
        assert m.check() == (binding.REC_OK, -1)
        got = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
        st = static(m.handle, d.data_ptr(), i.data_ptr(), l.data_ptr(), B, batch.nnz, got.data_ptr(),
                    fault.data_ptr(), stream)
        assert st == binding.REC_OK, binding.status_string(st)
        torch.cuda.synchronize()
        assert fault.tolist() == [binding.REC_OK, -1]
        assert torch.equal(got, want)
        if w.interaction == "concat":
            exact = orc.forward_towers(batch.dense, tabs, batch.indices, batch.lengths, bottom, top)
            mirror = orc.forward_towers(batch.dense, tabs, batch.indices, batch.lengths, bottom, top,
                                        orc.BF16_MIRROR)
        else:
            exact = orc.forward(batch.dense, tabs, batch.indices, batch.lengths, bottom, top)
            mirror = orc.forward(batch.dense, tabs, batch.indices, batch.lengths, bottom, top, orc.BF16_MIRROR)
        H.check_logits(got.cpu().numpy(), exact["logits"], mirror["logits"])
    m.close()


def test_static_scratch_reports_faults_and_rejects_what_does_not_fit(binding):
    print("static forward: faults and capacity", flush=True)
    static = _raw_static(binding)
    w = synth.WORKLOADS["tiny"].with_batch(64)
    m, _, _ = H.make_workload_model(binding, w)
    batch = synth.draw_batch(w, 3)
    bad = batch.indices.copy()
    bad[1234] = w.rows                       # one id past its table
    d, i, l = _dev(synth.Batch(batch.dense, bad, batch.lengths))
    out = torch.empty(64, dtype=torch.float32, device="cuda")
    fault = torch.zeros(2, dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    assert static(m.handle, d.data_ptr(), i.data_ptr(), l.data_ptr(), 64, bad.size, out.data_ptr(),
                  fault.data_ptr(), stream) == binding.REC_OK
    torch.cuda.synchronize()
    assert fault.tolist() == [binding.REC_ERR_INDEX_RANGE, 1234]
    assert m.check() == (binding.REC_OK, -1)      # the bound workspace's record is untouched
    # the next call starts from a clean record
    d, i, l = _dev(batch)
    assert static(m.handle, d.data_ptr(), i.data_ptr(), l.data_ptr(), 64, batch.nnz, out.data_ptr(),
                  fault.data_ptr(), stream) == binding.REC_OK
    torch.cuda.synchronize()
    assert fault.tolist() == [binding.REC_OK, -1]
    assert torch.isfinite(out).all()
    # a batch of zero samples runs no stage and still reports a clean record
    fault.fill_(7)
    assert static(m.handle, d.data_ptr(), i.data_ptr(), l.data_ptr(), 0, 0, out.data_ptr(),
                  fault.data_ptr(), stream) == binding.REC_OK
    torch.cuda.synchronize()
    assert fault.tolist() == [binding.REC_OK, -1]
    # host-checkable faults are refused as in rec_forward
    assert static(m.handle, d.data_ptr(), i.data_ptr(), l.data_ptr(), 65, batch.nnz, out.data_ptr(),
                  None, stream) == binding.REC_ERR_ARG
    assert static(m.handle, None, i.data_ptr(), l.data_ptr(), 64, batch.nnz, out.data_ptr(),
                  None, stream) == binding.REC_ERR_ARG
    m.close()
    # a batch whose intermediates exceed the static array is refused, nothing is enqueued
    big = synth.WORKLOADS["tiny"].with_batch(1 << 17)
    mb = binding.RecModel(big.num_tables, big.emb_dim, [1000] * big.num_tables, "f32", big.num_dense,
                          list(big.bottom), list(big.top), big.batch, big.batch * big.num_tables)
    for t in range(big.num_tables):
        mb.load_table(t, torch.zeros((1000, big.emb_dim), device="cuda"))
    H.load_mlps(binding, mb, synth.draw_mlp(big, "bottom"), synth.draw_mlp(big, "top"))
    B = big.batch
    d = torch.zeros((B, big.num_dense), device="cuda")
    l = torch.ones(big.num_tables * B, dtype=torch.int32, device="cuda")
    i = torch.zeros(big.num_tables * B, dtype=torch.int32, device="cuda")
    out = torch.empty(B, dtype=torch.float32, device="cuda")
    assert static(mb.handle, d.data_ptr(), i.data_ptr(), l.data_ptr(), B, i.numel(), out.data_ptr(),
                  None, stream) == binding.REC_ERR_CAPACITY
    assert static(mb.handle, d.data_ptr(), i.data_ptr(), l.data_ptr(), 512, 512 * big.num_tables,
                  out.data_ptr(), None, stream) == binding.REC_OK
    torch.cuda.synchronize()
    mb.close()
