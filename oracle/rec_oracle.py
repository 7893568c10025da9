"""ctypes wrapper around the C oracle (rec_oracle.c).

TEST INFRASTRUCTURE ONLY: called by tests, by the smoke check and by the
CPU-baseline leg of the benchmark.  It imports nothing from the device
package and the device package imports nothing from here.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rec_oracle.c")
_LIB = os.path.join(_HERE, "librec_oracle.so")

F32, F16 = 0, 1
EXACT, BF16_MIRROR = 0, 1


_LIB_SAN = os.path.join(_HERE, "librec_oracle_san.so")
SANITIZE_ENV = "REC_ORACLE_SANITIZED"   # set (to 1): load the build below instead


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall",
                               "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def build_sanitized(force: bool = False) -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (any
    finding aborts the process).  A process that loads it must have gcc's
    libasan preloaded; tests/test_sanitizers.py runs the pin suite that way."""
    if force or not os.path.exists(_LIB_SAN) or os.path.getmtime(_LIB_SAN) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                               "-fno-omit-frame-pointer", "-o", _LIB_SAN, _SRC, "-lm"])
    return _LIB_SAN


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build_sanitized() if os.environ.get(SANITIZE_ENV) else build())
        _lib.oracle_half_to_double.restype = C.c_double
        _lib.oracle_half_to_double.argtypes = [C.c_uint16]
        _lib.oracle_round_bf16.restype = C.c_double
        _lib.oracle_round_bf16.argtypes = [C.c_double]
        _lib.oracle_sigmoid.restype = C.c_double
        _lib.oracle_sigmoid.argtypes = [C.c_double]
        _lib.oracle_pool.restype = C.c_int64
        _lib.oracle_set_threads.restype = C.c_int
        _lib.oracle_set_threads.argtypes = [C.c_int]
    return _lib


def set_threads(n: int) -> int:
    return int(lib().oracle_set_threads(int(n)))


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _dtype_code(tables: Sequence[np.ndarray]) -> int:
    dt = tables[0].dtype
    assert all(t.dtype == dt for t in tables)
    if dt == np.float16:
        return F16
    assert dt == np.float32
    return F32


def _ptr_array(arrs: Sequence[np.ndarray]):
    return (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def half_to_double(bits: int) -> float:
    return float(lib().oracle_half_to_double(int(bits)))


def round_bf16(x: float) -> float:
    return float(lib().oracle_round_bf16(float(x)))


def sigmoid(x: float) -> float:
    return float(lib().oracle_sigmoid(float(x)))


def offsets(lengths: np.ndarray) -> Tuple[np.ndarray, int, int]:
    """(offsets int64 [n+1], rc, first_bad)."""
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    off = np.empty(lengths.size + 1, dtype=np.int64)
    bad = C.c_int64(-1)
    rc = lib().oracle_offsets(_p(lengths), C.c_int64(lengths.size), _p(off), C.byref(bad))
    return off, int(rc), int(bad.value)


def pool(tables: Sequence[np.ndarray], indices: np.ndarray, lengths: np.ndarray,
         B: int, want_abs: bool = False):
    """(P fp64 [B, T, D], abs_sum or None, n_bad, first_bad)."""
    tables = [np.ascontiguousarray(t) for t in tables]
    T, D = len(tables), tables[0].shape[1]
    rows = np.array([t.shape[0] for t in tables], dtype=np.int64)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    assert lengths.size == T * B and int(np.maximum(lengths, 0).sum()) == indices.size
    P = np.empty((B, T, D), dtype=np.float64)
    A = np.empty((B, T, D), dtype=np.float64) if want_abs else None
    bad = C.c_int64(-1)
    nbad = lib().oracle_pool(_ptr_array(tables), C.c_int(_dtype_code(tables)), _p(rows),
                             C.c_int(T), C.c_int(D), C.c_int(B), _p(indices), _p(lengths),
                             _p(P), _p(A) if want_abs else None, C.byref(bad))
    return P, A, int(nbad), int(bad.value)


def fc(x: np.ndarray, W: np.ndarray, b: np.ndarray, relu: bool, mode: int = EXACT) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    W = np.ascontiguousarray(W, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    B, n_in = x.shape
    n_out = W.shape[0]
    assert W.shape == (n_out, n_in) and b.shape == (n_out,)
    y = np.empty((B, n_out), dtype=np.float64)
    lib().oracle_fc(_p(x), _p(W), _p(b), C.c_int(B), C.c_int(n_in), C.c_int(n_out),
                    C.c_int(int(relu)), C.c_int(mode), _p(y))
    return y


def gram(x0: np.ndarray, P: np.ndarray) -> np.ndarray:
    x0 = np.ascontiguousarray(x0, dtype=np.float64)
    P = np.ascontiguousarray(P, dtype=np.float64)
    B, T, D = P.shape
    assert x0.shape == (B, D)
    Z = np.empty((B, T + 1, T + 1), dtype=np.float64)
    lib().oracle_gram(_p(x0), _p(P), C.c_int(B), C.c_int(T), C.c_int(D), _p(Z))
    return Z


def interact(x0: np.ndarray, P: np.ndarray) -> np.ndarray:
    x0 = np.ascontiguousarray(x0, dtype=np.float64)
    P = np.ascontiguousarray(P, dtype=np.float64)
    B, T, D = P.shape
    assert x0.shape == (B, D)
    out = np.empty((B, D + T * (T + 1) // 2), dtype=np.float64)
    lib().oracle_interact(_p(x0), _p(P), C.c_int(B), C.c_int(T), C.c_int(D), _p(out))
    return out


def forward(dense: np.ndarray, tables: Sequence[np.ndarray], indices: np.ndarray,
            lengths: np.ndarray, bottom: List[Tuple[np.ndarray, np.ndarray]],
            top: List[Tuple[np.ndarray, np.ndarray]], mode: int = EXACT) -> dict:
    """Whole forward.  Returns pooled, bottom_out, interact, logits (fp64)."""
    dense = np.ascontiguousarray(dense, dtype=np.float32)
    tables = [np.ascontiguousarray(t) for t in tables]
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    B, F = dense.shape
    T, D = len(tables), tables[0].shape[1]
    assert lengths.size == T * B and int(np.maximum(lengths, 0).sum()) == indices.size
    rows = np.array([t.shape[0] for t in tables], dtype=np.int64)

    def widths(layers, first):
        w = [first] + [L[0].shape[0] for L in layers]
        for i, (W, b) in enumerate(layers):
            assert W.shape == (w[i + 1], w[i]) and b.shape == (w[i + 1],)
        return np.array(w, dtype=np.int32)

    bw = widths(bottom, F)
    tw = widths(top, top[0][0].shape[1])
    bW = [np.ascontiguousarray(W, dtype=np.float32) for W, _ in bottom]
    bb = [np.ascontiguousarray(b, dtype=np.float32) for _, b in bottom]
    tW = [np.ascontiguousarray(W, dtype=np.float32) for W, _ in top]
    tb = [np.ascontiguousarray(b, dtype=np.float32) for _, b in top]
    width = D + T * (T + 1) // 2
    out = {
        "pooled": np.empty((B, T, D), dtype=np.float64),
        "bottom_out": np.empty((B, D), dtype=np.float64),
        "interact": np.empty((B, width), dtype=np.float64),
        "logits": np.empty(B, dtype=np.float64),
    }
    rc = lib().oracle_forward(
        _p(dense), _ptr_array(tables), C.c_int(_dtype_code(tables)), _p(rows),
        C.c_int(T), C.c_int(D), C.c_int(B), _p(indices), _p(lengths),
        C.c_int(len(bottom)), _p(bw), _ptr_array(bW), _ptr_array(bb),
        C.c_int(len(top)), _p(tw), _ptr_array(tW), _ptr_array(tb),
        C.c_int(mode), _p(out["pooled"]), _p(out["bottom_out"]), _p(out["interact"]),
        _p(out["logits"]))
    if rc != 0:
        raise ValueError("layer widths do not fit the model")
    return out


def concat(x0: np.ndarray, P: np.ndarray) -> np.ndarray:
    x0 = np.ascontiguousarray(x0, dtype=np.float64)
    P = np.ascontiguousarray(P, dtype=np.float64)
    B, T, D = P.shape
    w0 = x0.shape[1]
    assert x0.shape == (B, w0)
    out = np.empty((B, w0 + T * D), dtype=np.float64)
    lib().oracle_concat(_p(x0), C.c_int(w0), _p(P), C.c_int(B), C.c_int(T), C.c_int(D), _p(out))
    return out


def forward_towers(dense: np.ndarray, tables: Sequence[np.ndarray], indices: np.ndarray,
                   lengths: np.ndarray, bottom: List[Tuple[np.ndarray, np.ndarray]],
                   towers: List[List[Tuple[np.ndarray, np.ndarray]]], mode: int = EXACT) -> dict:
    """Concatenation model with len(towers) Predict-FC towers (`bottom` may be
    empty).  Returns pooled, bottom_out, concat, logits [B, n_towers] (fp64)."""
    dense = np.ascontiguousarray(dense, dtype=np.float32)
    tables = [np.ascontiguousarray(t) for t in tables]
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    B, F = dense.shape
    T, D = len(tables), tables[0].shape[1]
    assert lengths.size == T * B and int(np.maximum(lengths, 0).sum()) == indices.size
    rows = np.array([t.shape[0] for t in tables], dtype=np.int64)

    def widths(layers, first):
        w = [first] + [L[0].shape[0] for L in layers]
        for i, (W, b) in enumerate(layers):
            assert W.shape == (w[i + 1], w[i]) and b.shape == (w[i + 1],)
        return np.array(w, dtype=np.int32)

    bw = widths(bottom, F)
    w0 = int(bw[-1])
    width = w0 + T * D
    tw = widths(towers[0], towers[0][0][0].shape[1])
    for tower in towers:
        assert len(tower) == len(towers[0]) and np.array_equal(widths(tower, int(tw[0])), tw)
    bW = [np.ascontiguousarray(W, dtype=np.float32) for W, _ in bottom]
    bb = [np.ascontiguousarray(b, dtype=np.float32) for _, b in bottom]
    tW = [np.ascontiguousarray(W, dtype=np.float32) for tower in towers for W, _ in tower]
    tb = [np.ascontiguousarray(b, dtype=np.float32) for tower in towers for _, b in tower]
    out = {
        "pooled": np.empty((B, T, D), dtype=np.float64),
        "bottom_out": np.empty((B, w0), dtype=np.float64),
        "concat": np.empty((B, width), dtype=np.float64),
        "logits": np.empty((B, len(towers)), dtype=np.float64),
    }
    rc = lib().oracle_forward_towers(
        _p(dense), _ptr_array(tables), C.c_int(_dtype_code(tables)), _p(rows),
        C.c_int(T), C.c_int(D), C.c_int(B), _p(indices), _p(lengths),
        C.c_int(len(bottom)), _p(bw), _ptr_array(bW), _ptr_array(bb),
        C.c_int(len(towers)), C.c_int(len(towers[0])), _p(tw), _ptr_array(tW), _ptr_array(tb),
        C.c_int(mode), _p(out["pooled"]), _p(out["bottom_out"]), _p(out["concat"]),
        _p(out["logits"]))
    if rc != 0:
        raise ValueError("layer widths do not fit the model")
    return out
