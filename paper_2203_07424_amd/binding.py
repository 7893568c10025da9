"""ctypes binding of the C boundary declared in include/rec.h.

Argument marshalling only: every step of the forward pass runs in the HIP
library.  PyTorch supplies device memory and the stream.  Importing this
module raises if the library has not been built; there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import torch  # loads the HIP runtime the library binds to

_PKG = os.path.dirname(os.path.abspath(__file__))
# REC_MI355X_LIBRARY: another build of the same library (the host-instrumented
# one of build.build_host_sanitized()); unset in normal use.
LIB_PATH = os.environ.get("REC_MI355X_LIBRARY") or os.path.join(_PKG, "librec_mi355x.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -m paper_2203_07424_amd.build "
        "or __graft_entry__.build()); there is no CPU fallback")

_lib = C.CDLL(LIB_PATH)

REC_OK = 0
REC_ERR_ARG, REC_ERR_SHAPE, REC_ERR_STATE, REC_ERR_LENGTHS = 1, 2, 3, 4
REC_ERR_INDEX_RANGE, REC_ERR_OVERFLOW, REC_ERR_DEVICE, REC_ERR_CAPACITY = 5, 6, 7, 8
REC_STATIC_SCRATCH_BYTES = 64 << 20
REC_STATIC_MAX_TABLES = 64
REC_F32, REC_F16 = 0, 1
REC_BOTTOM, REC_TOP = 0, 1          # REC_TOP + k: tower k of the Predict-FC
REC_INTERACT_DOT, REC_INTERACT_CONCAT = 0, 1
REC_MAX_TOWERS = 8
REC_DBG_OFFSETS, REC_DBG_POOLED, REC_DBG_BOTTOM_OUT, REC_DBG_INTERACT = 0, 1, 2, 3
REC_OPT_OVERLAP_DENSE = 0
REC_OPT_STREAM_ROWS = 1
REC_OPT_FUSE_MLP = 2
REC_OPT_PIPELINE = 3
REC_NUM_STAGES = 7
STAGE_NAMES = ("scan", "pool", "bottom_first", "bottom_rest", "interact", "top_first", "top_rest")

EXPORTS = ("rec_create", "rec_destroy", "rec_workspace_bytes", "rec_bind_workspace",
           "rec_load_tables", "rec_load_hot_rows", "rec_mlp_packed_bytes", "rec_load_mlp", "rec_forward", "rec_forward_static", "rec_check",
           "rec_debug_get", "rec_set_option", "rec_set_dense_stream", "rec_set_pool_streams", "rec_drain", "rec_set_profiling", "rec_stage_ms", "rec_status_string",
           "rec_synth_fill_table", "rec_probe_mfma")


class rec_config(C.Structure):
    _fields_ = [("num_tables", C.c_int32), ("emb_dim", C.c_int32),
                ("rows", C.POINTER(C.c_int64)), ("table_dtype", C.c_int32),
                ("num_dense", C.c_int32), ("n_bottom", C.c_int32),
                ("bottom_widths", C.POINTER(C.c_int32)), ("n_top", C.c_int32),
                ("top_widths", C.POINTER(C.c_int32)), ("max_batch", C.c_int32),
                ("max_nnz", C.c_int64), ("interaction", C.c_int32), ("num_towers", C.c_int32)]


_vp = C.c_void_p
_lib.rec_create.restype = C.c_int
_lib.rec_create.argtypes = [C.POINTER(rec_config), C.POINTER(_vp)]
_lib.rec_destroy.restype = None
_lib.rec_destroy.argtypes = [_vp]
_lib.rec_workspace_bytes.restype = C.c_size_t
_lib.rec_workspace_bytes.argtypes = [_vp]
_lib.rec_bind_workspace.restype = C.c_int
_lib.rec_bind_workspace.argtypes = [_vp, _vp, C.c_size_t, _vp]
_lib.rec_load_tables.restype = C.c_int
_lib.rec_load_tables.argtypes = [_vp, C.c_int32, _vp]
_lib.rec_load_hot_rows.restype = C.c_int
_lib.rec_load_hot_rows.argtypes = [_vp, C.c_int32, _vp, C.c_int32]
_lib.rec_mlp_packed_bytes.restype = C.c_size_t
_lib.rec_mlp_packed_bytes.argtypes = [_vp, C.c_int32, C.c_int32]
_lib.rec_load_mlp.restype = C.c_int
_lib.rec_load_mlp.argtypes = [_vp, C.c_int32, C.c_int32, _vp, _vp, _vp, _vp]
_lib.rec_forward.restype = C.c_int
_lib.rec_forward.argtypes = [_vp, _vp, _vp, _vp, C.c_int32, C.c_int64, _vp, _vp]
_lib.rec_forward_static.restype = C.c_int
_lib.rec_forward_static.argtypes = [_vp, _vp, _vp, _vp, C.c_int32, C.c_int64, _vp, _vp, _vp]
_lib.rec_check.restype = C.c_int
_lib.rec_check.argtypes = [_vp, _vp, C.POINTER(C.c_int64)]
_lib.rec_debug_get.restype = C.c_int
_lib.rec_debug_get.argtypes = [_vp, C.c_int32, C.POINTER(_vp), C.POINTER(C.c_int64)]
_lib.rec_set_option.restype = C.c_int
_lib.rec_set_option.argtypes = [_vp, C.c_int32, C.c_int32]
_lib.rec_set_dense_stream.restype = C.c_int
_lib.rec_set_dense_stream.argtypes = [_vp, _vp]
_lib.rec_set_pool_streams.restype = C.c_int
_lib.rec_set_pool_streams.argtypes = [_vp, _vp, _vp]
_lib.rec_drain.restype = C.c_int
_lib.rec_drain.argtypes = [_vp, _vp]
_lib.rec_set_profiling.restype = C.c_int
_lib.rec_set_profiling.argtypes = [_vp, C.c_int32, C.c_int32]
_lib.rec_stage_ms.restype = C.c_int
_lib.rec_stage_ms.argtypes = [_vp, C.c_int32, C.POINTER(C.c_float)]
_lib.rec_status_string.restype = C.c_char_p
_lib.rec_status_string.argtypes = [C.c_int]
_lib.rec_synth_fill_table.restype = C.c_int
_lib.rec_synth_fill_table.argtypes = [_vp, C.c_int32, C.c_uint64, C.c_int32, C.c_int64, C.c_int32, _vp]


_lib.rec_probe_mfma.restype = C.c_int
_lib.rec_probe_mfma.argtypes = [C.c_int32, C.c_int32, C.c_int32, _vp, _vp]


class RecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def status_string(status: int) -> str:
    return _lib.rec_status_string(int(status)).decode()


def _stream() -> Optional[int]:
    # Without a device only the host-side argument checks of the library can
    # run, and those never touch the stream.
    if not torch.cuda.is_available():
        return None
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


# Raw entry points, same names as the C boundary; each returns the status.
def rec_create(num_tables: int, emb_dim: int, rows: Sequence[int], table_dtype: int,
               num_dense: int, bottom_widths: Sequence[int], top_widths: Sequence[int],
               max_batch: int, max_nnz: int, interaction: int = REC_INTERACT_DOT,
               num_towers: int = 1) -> Tuple[int, Optional[int]]:
    rows_a = (C.c_int64 * len(rows))(*rows)
    bw = (C.c_int32 * len(bottom_widths))(*bottom_widths)
    tw = (C.c_int32 * len(top_widths))(*top_widths)
    cfg = rec_config(num_tables, emb_dim, rows_a, table_dtype, num_dense, len(bottom_widths) - 1,
                     bw, len(top_widths) - 1, tw, max_batch, max_nnz, interaction, num_towers)
    out = _vp()
    st = _lib.rec_create(C.byref(cfg), C.byref(out))
    return st, out.value


def rec_destroy(m: int) -> None:
    _lib.rec_destroy(m)


def rec_workspace_bytes(m: int) -> int:
    return int(_lib.rec_workspace_bytes(m))


def rec_bind_workspace(m: int, ws: torch.Tensor) -> int:
    return _lib.rec_bind_workspace(m, ws.data_ptr(), ws.numel() * ws.element_size(), _stream())


def rec_load_tables(m: int, table: int, dev_rows: torch.Tensor) -> int:
    return _lib.rec_load_tables(m, table, dev_rows.data_ptr())


def rec_load_hot_rows(m: int, table: int, dev_ids: Optional[torch.Tensor]) -> int:
    n = 0 if dev_ids is None else dev_ids.numel()
    return _lib.rec_load_hot_rows(m, table, _ptr(dev_ids), n)


def rec_mlp_packed_bytes(m: int, which: int, layer: int) -> int:
    return int(_lib.rec_mlp_packed_bytes(m, which, layer))


def rec_load_mlp(m: int, which: int, layer: int, dev_W: torch.Tensor, dev_b: torch.Tensor,
                 dev_packed: torch.Tensor) -> int:
    return _lib.rec_load_mlp(m, which, layer, dev_W.data_ptr(), dev_b.data_ptr(),
                             dev_packed.data_ptr(), _stream())


def rec_forward(m: int, dev_dense, dev_indices, dev_lengths, batch: int, nnz: int, dev_logits) -> int:
    return _lib.rec_forward(m, _ptr(dev_dense), _ptr(dev_indices), _ptr(dev_lengths), batch, nnz,
                            _ptr(dev_logits), _stream())


def rec_forward_static(m: int, dev_dense, dev_indices, dev_lengths, batch: int, nnz: int, dev_logits,
                       dev_fault=None) -> int:
    return _lib.rec_forward_static(m, _ptr(dev_dense), _ptr(dev_indices), _ptr(dev_lengths), batch, nnz,
                                   _ptr(dev_logits), _ptr(dev_fault), _stream())


def rec_check(m: int) -> Tuple[int, int]:
    pos = C.c_int64(-1)
    st = _lib.rec_check(m, _stream(), C.byref(pos))
    return st, int(pos.value)


def rec_debug_get(m: int, what: int) -> Tuple[int, Optional[int], int]:
    p, ld = _vp(), C.c_int64(0)
    st = _lib.rec_debug_get(m, what, C.byref(p), C.byref(ld))
    return st, p.value, int(ld.value)


def rec_set_option(m: int, option: int, value: int) -> int:
    return _lib.rec_set_option(m, int(option), int(value))


def rec_set_dense_stream(m: int, stream: Optional["torch.cuda.Stream"]) -> int:
    return _lib.rec_set_dense_stream(m, None if stream is None else stream.cuda_stream)


def rec_set_pool_streams(m: int, a: Optional["torch.cuda.Stream"], b: Optional["torch.cuda.Stream"]) -> int:
    return _lib.rec_set_pool_streams(m, None if a is None else a.cuda_stream, None if b is None else b.cuda_stream)


def rec_drain(m: int) -> int:
    return _lib.rec_drain(m, _stream())


def rec_set_profiling(m: int, slots: int, period: int = 1) -> int:
    return _lib.rec_set_profiling(m, int(slots), int(period))


def rec_stage_ms(m: int, slot: int = 0) -> Tuple[int, List[float]]:
    ms = (C.c_float * REC_NUM_STAGES)()
    st = _lib.rec_stage_ms(m, slot, ms)
    return st, [float(v) for v in ms]


def rec_synth_fill_table(dev_rows: torch.Tensor, seed: int, table: int) -> int:
    dtype = REC_F16 if dev_rows.dtype == torch.float16 else REC_F32
    return _lib.rec_synth_fill_table(dev_rows.data_ptr(), dtype, seed, table, dev_rows.shape[0],
                                     dev_rows.shape[1], _stream())


def rec_probe_mfma(random_operands: bool, blocks: int, iters: int, dev_sink: Optional[torch.Tensor]) -> int:
    """One launch of nothing but bf16 matrix instructions (blocks * 8 * iters * 32 * 32768 flops)."""
    return _lib.rec_probe_mfma(int(bool(random_operands)), int(blocks), int(iters), _ptr(dev_sink), _stream())


class RecModel:
    """Owns the device buffers of one model and forwards batches through the library."""

    def __init__(self, num_tables: int, emb_dim: int, rows: Sequence[int], table_dtype: str,
                 num_dense: int, bottom_widths: Sequence[int], top_widths: Sequence[int],
                 max_batch: int, max_nnz: int, device: str = "cuda:0", interaction: str = "dot",
                 towers: int = 1, pipeline: bool = False,
                 dense_stream: Optional["torch.cuda.Stream"] = None,
                 pool_streams: Sequence[Optional["torch.cuda.Stream"]] = (None, None)):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the forward pass has no CPU path")
        self.device = torch.device(device)
        self.T, self.D, self.F = num_tables, emb_dim, num_dense
        self.table_dtype = {"f32": torch.float32, "f16": torch.float16}[table_dtype]
        self.width = top_widths[0]
        self.n_bottom, self.n_top = len(bottom_widths) - 1, len(top_widths) - 1
        self.towers, self.w0 = towers, bottom_widths[-1]
        code = REC_F16 if table_dtype == "f16" else REC_F32
        inter = {"dot": REC_INTERACT_DOT, "concat": REC_INTERACT_CONCAT}[interaction]
        st, self.handle = rec_create(num_tables, emb_dim, list(rows), code, num_dense,
                                     list(bottom_widths), list(top_widths), max_batch, max_nnz,
                                     inter, towers)
        if st != REC_OK:
            raise RecError(st, "rec_create")
        self.pipeline, self.dense_stream, self.pool_streams = bool(pipeline), dense_stream, tuple(pool_streams)
        if pipeline:      # decides the workspace size, so it is set before binding
            self._ok(rec_set_option(self.handle, REC_OPT_PIPELINE, 1), "rec_set_option")
            self._ok(rec_set_dense_stream(self.handle, dense_stream), "rec_set_dense_stream")
            self._ok(rec_set_pool_streams(self.handle, *self.pool_streams), "rec_set_pool_streams")
        self.ws = torch.empty(rec_workspace_bytes(self.handle), dtype=torch.uint8, device=self.device)
        self._ok(rec_bind_workspace(self.handle, self.ws), "rec_bind_workspace")
        self.tables: List[Optional[torch.Tensor]] = [None] * num_tables
        self.hot: List[Optional[torch.Tensor]] = [None] * num_tables
        self.packed: dict = {}
        self.last_batch = 0

    def _ok(self, st: int, where: str) -> None:
        if st != REC_OK:
            raise RecError(st, where)

    def close(self) -> None:
        if getattr(self, "handle", None):
            torch.cuda.synchronize(self.device)
            rec_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def load_table(self, t: int, dev_rows: torch.Tensor) -> None:
        assert dev_rows.is_cuda and dev_rows.is_contiguous() and dev_rows.dtype == self.table_dtype
        self._ok(rec_load_tables(self.handle, t, dev_rows), "rec_load_tables")
        self.tables[t] = dev_rows

    def load_hot_rows(self, t: int, ids) -> None:
        """ids: int32 row ids (tensor or array), or None / empty to remove the list."""
        dev_ids = None
        if ids is not None and len(ids) > 0:
            dev_ids = torch.as_tensor(ids, dtype=torch.int32).to(self.device).contiguous()
        self._ok(rec_load_hot_rows(self.handle, t, dev_ids), "rec_load_hot_rows")
        self.hot[t] = dev_ids

    def load_mlp(self, which: int, layer: int, W: torch.Tensor, b: torch.Tensor) -> None:
        W = W.to(self.device, torch.float32).contiguous()
        b = b.to(self.device, torch.float32).contiguous()
        packed = torch.empty(rec_mlp_packed_bytes(self.handle, which, layer), dtype=torch.uint8,
                             device=self.device)
        self._ok(rec_load_mlp(self.handle, which, layer, W, b, packed), "rec_load_mlp")
        torch.cuda.current_stream().synchronize()   # W and b may be freed after this
        self.packed[(which, layer)] = packed

    def forward(self, dense: torch.Tensor, indices: torch.Tensor, lengths: torch.Tensor,
                logits: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Returns fp32 logits: [batch] for one Predict-FC stack, [batch, towers] for several."""
        batch = dense.shape[0]
        if logits is None:
            shape = (batch,) if self.towers == 1 else (batch, self.towers)
            logits = torch.empty(shape, dtype=torch.float32, device=self.device)
        # The library sees pointers only: check here that every buffer is as large
        # as the call says, of the right type, contiguous and on the device.
        for name, t, dt, n in (("dense", dense, torch.float32, batch * self.F),
                               ("indices", indices, torch.int32, indices.numel()),
                               ("lengths", lengths, torch.int32, self.T * batch),
                               ("logits", logits, torch.float32, batch * self.towers)):
            if not (t.is_cuda and t.is_contiguous() and t.dtype == dt and t.numel() >= n):
                raise ValueError(f"rec_forward: {name} must be a contiguous {dt} device tensor of at least {n} elements")
        self._ok(rec_forward(self.handle, dense, indices, lengths, batch, indices.numel(), logits),
                 "rec_forward")
        self.last_batch = batch
        return logits

    def forward_static(self, dense: torch.Tensor, indices: torch.Tensor, lengths: torch.Tensor,
                       logits: torch.Tensor, fault: Optional[torch.Tensor] = None) -> torch.Tensor:
        """rec_forward_static(): the same pass with the library's static scratch; the
        caller brings every buffer (logits fp32, fault int64 [2] or None)."""
        batch = dense.shape[0]
        for name, t, dt, n in (("dense", dense, torch.float32, batch * self.F),
                               ("indices", indices, torch.int32, indices.numel()),
                               ("lengths", lengths, torch.int32, self.T * batch),
                               ("logits", logits, torch.float32, batch * self.towers)):
            if not (t.is_cuda and t.is_contiguous() and t.dtype == dt and t.numel() >= n):
                raise ValueError(f"rec_forward_static: {name} must be a contiguous {dt} device tensor of at least {n} elements")
        if fault is not None and not (fault.is_cuda and fault.dtype == torch.int64 and fault.numel() >= 2):
            raise ValueError("rec_forward_static: fault must be an int64 device tensor of 2 elements")
        self._ok(rec_forward_static(self.handle, dense, indices, lengths, batch, indices.numel(), logits, fault),
                 "rec_forward_static")
        return logits

    def check(self) -> Tuple[int, int]:
        return rec_check(self.handle)

    def drain(self) -> None:
        """Pipelined models: orders every forward enqueued so far on the current stream."""
        self._ok(rec_drain(self.handle), "rec_drain")

    def set_option(self, option: int, value: int) -> None:
        self._ok(rec_set_option(self.handle, option, value), "rec_set_option")

    def set_profiling(self, slots: int, period: int = 1) -> None:
        self._ok(rec_set_profiling(self.handle, slots, period), "rec_set_profiling")

    def stage_ms(self, slot: int = 0) -> dict:
        st, ms = rec_stage_ms(self.handle, slot)
        self._ok(st, "rec_stage_ms")
        return dict(zip(STAGE_NAMES, ms))

    def _view(self, what: int, nbytes: int) -> Tuple[torch.Tensor, int]:
        st, p, ld = rec_debug_get(self.handle, what)
        self._ok(st, "rec_debug_get")
        off = p - self.ws.data_ptr()
        return self.ws[off:off + nbytes], ld

    def debug_offsets(self) -> torch.Tensor:
        n = self.T * self.last_batch + 1
        raw, _ = self._view(REC_DBG_OFFSETS, 4 * n)
        return raw.view(torch.int32).clone()

    def debug_pooled(self) -> torch.Tensor:
        B = self.last_batch
        raw, _ = self._view(REC_DBG_POOLED, 4 * B * self.T * self.D)
        return raw.view(torch.float32).view(B, self.T, self.D).clone()

    def debug_bottom_out(self) -> torch.Tensor:
        B = self.last_batch
        st, p, ld = rec_debug_get(self.handle, REC_DBG_BOTTOM_OUT)
        raw, ld = self._view(REC_DBG_BOTTOM_OUT, 4 * B * ld)
        return raw.view(torch.float32).view(B, ld)[:, :self.w0].clone()

    def debug_interact(self) -> torch.Tensor:
        """The Predict-FC input, bf16 [B, ld]; columns beyond its width are zero padding."""
        B = self.last_batch
        st, p, ld = rec_debug_get(self.handle, REC_DBG_INTERACT)
        raw, ld = self._view(REC_DBG_INTERACT, 2 * B * ld)
        return raw.view(torch.bfloat16).view(B, ld).clone()


class CapturedForward:
    """One or more forwards recorded into a HIP graph and replayed with a single launch.

    rec_forward() only enqueues kernels (no allocation, no synchronisation, no
    memset), so it can be recorded under stream capture.  The graph replays the
    recorded pointers: callers keep `batches` and `logits` alive and refresh
    their contents in place.  Stage events must be off while recording."""

    def __init__(self, model: RecModel, batches, logits):
        self.model, self.batches, self.logits = model, list(batches), list(logits)
        assert len(self.batches) == len(self.logits) and self.batches
        for (d, i, l), out in zip(self.batches, self.logits):   # warm-up outside capture
            model.forward(d, i, l, out)
        model.drain()
        torch.cuda.synchronize(model.device)
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            for (d, i, l), out in zip(self.batches, self.logits):
                model.forward(d, i, l, out)
            model.drain()       # a pipelined model's other streams join the capture here

    def replay(self) -> None:
        self.graph.replay()
