"""Host-side checks of the C boundary that need no GPU: the library loads,
exports every declared symbol, and validates shapes and call order."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2203_07424_amd import binding as b
    return b


def declared_symbols():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        with open(os.path.join(ROOT, "include", fn)) as f:
            names += re.findall(r"REC_API[^;(]*?\b(rec_\w+)\s*\(", f.read())
    return names


def test_library_exports_every_declared_symbol(binding):
    names = declared_symbols()
    assert len(names) >= 14 and "rec_forward" in names and "rec_synth_fill_table" in names
    lib = C.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(names) == sorted(binding.EXPORTS)


def test_status_strings(binding):
    seen = {binding.status_string(s) for s in range(8)}
    assert len(seen) == 8 and binding.status_string(0) == "ok"
    assert binding.status_string(99) == "unknown status"


def _create(b, **kw):
    a = dict(num_tables=2, emb_dim=8, rows=[10, 20], table_dtype=b.REC_F32, num_dense=4,
             bottom_widths=[4, 16, 8], top_widths=[8 + 3, 5, 1], max_batch=32, max_nnz=1000)
    a.update(kw)
    return b.rec_create(**a)


def test_create_validates_shapes(binding):
    b = binding
    st, h = _create(b)
    assert st == b.REC_OK and h
    assert b.rec_workspace_bytes(h) > 0 and b.rec_workspace_bytes(h) % 256 == 0
    assert b.rec_mlp_packed_bytes(h, b.REC_BOTTOM, 0) >= 64 * 64 * 2 + 64 * 4
    assert b.rec_mlp_packed_bytes(h, b.REC_BOTTOM, 2) == 0
    assert b.rec_mlp_packed_bytes(h, 7, 0) == 0
    b.rec_destroy(h)
    assert _create(b, bottom_widths=[4, 16, 7])[0] == b.REC_ERR_SHAPE      # must end in D
    assert _create(b, bottom_widths=[5, 16, 8])[0] == b.REC_ERR_SHAPE      # must start at F
    assert _create(b, top_widths=[12, 5, 1])[0] == b.REC_ERR_SHAPE         # D + T(T+1)/2 = 11
    assert _create(b, top_widths=[11, 5, 2])[0] == b.REC_ERR_SHAPE         # one logit
    assert _create(b, emb_dim=6, bottom_widths=[4, 6], top_widths=[9, 1])[0] == b.REC_ERR_SHAPE
    assert _create(b, emb_dim=12, bottom_widths=[4, 12], top_widths=[15, 1])[0] == b.REC_ERR_SHAPE
    assert _create(b, rows=[10, 2 ** 31])[0] == b.REC_ERR_OVERFLOW
    assert _create(b, max_nnz=2 ** 31)[0] == b.REC_ERR_OVERFLOW
    assert _create(b, max_batch=2 ** 30)[0] == b.REC_ERR_OVERFLOW
    assert _create(b, rows=[10, 0])[0] == b.REC_ERR_ARG
    assert _create(b, max_batch=0)[0] == b.REC_ERR_ARG
    assert _create(b, table_dtype=5)[0] == b.REC_ERR_ARG
    # fp16 rows of 8 elements are exactly 16 bytes: allowed
    st, h = _create(b, table_dtype=b.REC_F16)
    assert st == b.REC_OK
    b.rec_destroy(h)


def test_concat_and_tower_shapes(binding):
    ok = dict(num_tables=2, emb_dim=8, rows=[10, 10], table_dtype=binding.REC_F32, num_dense=4,
              max_batch=4, max_nnz=100)
    # concat: first Predict-FC width must be w0 + T * D
    st, h = binding.rec_create(bottom_widths=[4], top_widths=[4 + 16, 8, 1],
                               interaction=binding.REC_INTERACT_CONCAT, num_towers=2, **ok)
    assert st == binding.REC_OK
    assert binding.rec_mlp_packed_bytes(h, binding.REC_TOP + 1, 0) > 0
    assert binding.rec_mlp_packed_bytes(h, binding.REC_TOP + 2, 0) == 0      # no such tower
    assert binding.rec_mlp_packed_bytes(h, binding.REC_BOTTOM, 0) == 0       # no Bottom-FC
    binding.rec_destroy(h)
    st, _ = binding.rec_create(bottom_widths=[4], top_widths=[8 + 3, 8, 1],
                               interaction=binding.REC_INTERACT_CONCAT, num_towers=1, **ok)
    assert st == binding.REC_ERR_SHAPE
    st, _ = binding.rec_create(bottom_widths=[4], top_widths=[20, 1], interaction=2, num_towers=1, **ok)
    assert st == binding.REC_ERR_ARG
    st, _ = binding.rec_create(bottom_widths=[4], top_widths=[20, 1], interaction=binding.REC_INTERACT_CONCAT,
                               num_towers=binding.REC_MAX_TOWERS + 1, **ok)
    assert st == binding.REC_ERR_ARG
    # pairwise dots without a Bottom-FC need num_dense = emb_dim
    st, _ = binding.rec_create(bottom_widths=[4], top_widths=[8 + 3, 1], **ok)
    assert st == binding.REC_ERR_SHAPE


def test_null_and_order_errors_without_device(binding):
    b = binding
    lib = C.CDLL(b.LIB_PATH)
    lib.rec_create.restype = C.c_int
    assert lib.rec_create(None, None) == b.REC_ERR_ARG
    st, h = _create(b)
    assert st == b.REC_OK
    lib.rec_forward.restype = C.c_int
    lib.rec_forward.argtypes = [C.c_void_p] * 4 + [C.c_int32, C.c_int64, C.c_void_p, C.c_void_p]
    # nothing bound or loaded yet
    assert lib.rec_forward(h, None, None, None, 4, 10, None, None) == b.REC_ERR_STATE
    assert lib.rec_forward(h, None, None, None, 33, 10, None, None) == b.REC_ERR_ARG    # > max_batch
    assert lib.rec_forward(h, None, None, None, 4, 1001, None, None) == b.REC_ERR_ARG   # > max_nnz
    assert lib.rec_forward(h, None, None, None, -1, 0, None, None) == b.REC_ERR_ARG
    assert lib.rec_forward(None, None, None, None, 1, 0, None, None) == b.REC_ERR_ARG
    lib.rec_load_tables.restype = C.c_int
    lib.rec_load_tables.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    assert lib.rec_load_tables(h, 0, 4096) == b.REC_ERR_STATE       # no workspace yet
    assert lib.rec_load_tables(h, 2, 4096) == b.REC_ERR_ARG         # table id
    assert lib.rec_load_tables(h, 0, 4100) == b.REC_ERR_ARG         # not 16-byte aligned
    assert b.rec_check(h)[0] == b.REC_ERR_STATE
    assert b.rec_debug_get(h, b.REC_DBG_POOLED)[0] == b.REC_ERR_STATE
    assert b.rec_stage_ms(h)[0] == b.REC_ERR_STATE
    assert b.rec_set_profiling(h, 4, 0) == b.REC_ERR_ARG
    assert b.rec_set_option(h, 99, 1) == b.REC_ERR_ARG
    assert b.rec_set_option(h, b.REC_OPT_FUSE_MLP, 3) == b.REC_ERR_ARG
    assert b.rec_set_option(h, b.REC_OPT_FUSE_MLP, 2) == b.REC_OK
    lib.rec_bind_workspace.restype = C.c_int
    lib.rec_bind_workspace.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    assert lib.rec_bind_workspace(h, None, 1 << 20, None) == b.REC_ERR_ARG
    assert lib.rec_bind_workspace(h, 4096, 16, None) == b.REC_ERR_ARG       # too small
    assert lib.rec_bind_workspace(h, 4100, 1 << 30, None) == b.REC_ERR_ARG  # misaligned
    b.rec_destroy(h)
    b.rec_destroy(None)
    # the matrix-rate probe checks its arguments before touching the device
    assert b.rec_probe_mfma(True, 256, 100, None) == b.REC_ERR_ARG
    lib.rec_probe_mfma.restype = C.c_int
    lib.rec_probe_mfma.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    assert lib.rec_probe_mfma(1, 0, 100, 4096, None) == b.REC_ERR_ARG
    assert lib.rec_probe_mfma(1, 256, 0, 4096, None) == b.REC_ERR_ARG
    assert lib.rec_probe_mfma(1, 1 << 20, 1, 4096, None) == b.REC_ERR_ARG
