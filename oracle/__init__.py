"""Python face of the CPU oracle (``moe_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's cpu_baseline leg.  The HIP library and its binding never import it.

All arrays are numpy, on the host.  bf16 tensors travel as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")

BF16, F32, F64 = 0, 1, 2
SOFTMAX_TOPK, SIGMOID_TOPK = 0, 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (contraction off, explicit fmaf only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-mfma", "-fopenmp",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_logit_r64.restype = ctypes.c_float
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float64:
        return F64
    raise TypeError(f"unsupported dtype {a.dtype}")


def _c(a, dtype=None):
    return np.ascontiguousarray(a, dtype=dtype)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def logits(x: np.ndarray, W_r: np.ndarray, bias: np.ndarray | None) -> np.ndarray:
    """fp32 router logits [N,E] in the canonical R64 summation order."""
    x = _c(x)
    W_r = _c(W_r, np.float32)
    N, H = x.shape
    E = W_r.shape[1]
    assert W_r.shape[0] == H
    b = None if bias is None else _c(bias, np.float32)
    out = np.empty((N, E), dtype=np.float32)
    _load().oracle_logits(_p(x), _dt(x), ctypes.c_int64(N), ctypes.c_int64(H), _p(W_r), _p(b),
                          ctypes.c_int(E), _p(out))
    return out


def topk(lg: np.ndarray, K: int, score_mode: int):
    """(topk_idx int32 [N,K], topk_w float64 [N,K]) from fp32 logits [N,E]."""
    lg = _c(lg, np.float32)
    N, E = lg.shape
    assert 1 <= K <= E
    idx = np.empty((N, K), dtype=np.int32)
    w = np.empty((N, K), dtype=np.float64)
    _load().oracle_topk(_p(lg), ctypes.c_int64(N), ctypes.c_int(E), ctypes.c_int(K),
                        ctypes.c_int(score_mode), _p(idx), _p(w))
    return idx, w


def route(x, W_r, bias, K: int, score_mode: int):
    lg = logits(x, W_r, bias)
    idx, w = topk(lg, K, score_mode)
    return idx, w, lg


def layout(topk_idx: np.ndarray, E: int, G: int) -> dict:
    topk_idx = _c(topk_idx, np.int32)
    N, K = topk_idx.shape
    assert E % G == 0
    assert topk_idx.size == 0 or (topk_idx.min() >= 0 and topk_idx.max() < E)
    R = N * K
    out = dict(
        expert_counts=np.empty(E, np.int32), expert_offsets=np.empty(E + 1, np.int32),
        dest_counts=np.empty(G, np.int32), dest_offsets=np.empty(G + 1, np.int32),
        slot_of_row=np.empty(R, np.int32), row_of_slot=np.empty(R, np.int32))
    _load().oracle_layout(_p(topk_idx), ctypes.c_int64(N), ctypes.c_int(K), ctypes.c_int(E),
                          ctypes.c_int(G), _p(out["expert_counts"]), _p(out["expert_offsets"]),
                          _p(out["dest_counts"]), _p(out["dest_offsets"]),
                          _p(out["slot_of_row"]), _p(out["row_of_slot"]))
    return out


def layout_arrival(topk_idx: np.ndarray, E: int, G: int, arrival: np.ndarray) -> dict:
    """Layout with rows packed in the order `arrival` lists them (flat rows, a permutation)."""
    topk_idx = _c(topk_idx, np.int32)
    N, K = topk_idx.shape
    R = N * K
    arrival = _c(arrival, np.int32)
    assert E % G == 0 and arrival.shape == (R,)
    assert np.array_equal(np.sort(arrival), np.arange(R, dtype=np.int32))
    assert topk_idx.size == 0 or (topk_idx.min() >= 0 and topk_idx.max() < E)
    out = dict(
        expert_counts=np.empty(E, np.int32), expert_offsets=np.empty(E + 1, np.int32),
        dest_counts=np.empty(G, np.int32), dest_offsets=np.empty(G + 1, np.int32),
        slot_of_row=np.empty(R, np.int32), row_of_slot=np.empty(R, np.int32))
    _load().oracle_layout_arrival(_p(topk_idx), ctypes.c_int64(N), ctypes.c_int(K), ctypes.c_int(E),
                                  ctypes.c_int(G), _p(arrival), _p(out["expert_counts"]),
                                  _p(out["expert_offsets"]), _p(out["dest_counts"]),
                                  _p(out["dest_offsets"]), _p(out["slot_of_row"]), _p(out["row_of_slot"]))
    return out


def permute(x: np.ndarray, K: int, slot_of_row: np.ndarray) -> np.ndarray:
    x = _c(x)
    N, H = x.shape
    slot_of_row = _c(slot_of_row, np.int32)
    assert slot_of_row.size == N * K
    xp = np.empty((N * K, H), dtype=x.dtype)
    _load().oracle_permute(_p(x), ctypes.c_int64(H * x.itemsize), ctypes.c_int64(N),
                           ctypes.c_int(K), _p(slot_of_row), _p(xp))
    return xp


def ffn_rows(xp, seg_offsets, W_gate, W_up, W_down, rows=None) -> np.ndarray:
    """fp64 SwiGLU expert outputs for `rows` of xp (all rows when None).
    W_gate, W_up: [E_local, F, H];  W_down: [E_local, H, F]."""
    xp = _c(xp)
    W_gate, W_up, W_down = _c(W_gate), _c(W_up), _c(W_down)
    M, H = xp.shape
    E_local, F, H2 = W_gate.shape
    assert H2 == H and W_up.shape == W_gate.shape and W_down.shape == (E_local, H, F)
    assert W_gate.dtype == W_up.dtype == W_down.dtype
    seg_offsets = _c(seg_offsets, np.int32)
    assert seg_offsets.size == E_local + 1
    if rows is None:
        r, nrows = None, M
    else:
        r = _c(rows, np.int64)
        nrows = r.size
        assert nrows == 0 or (r.min() >= 0 and r.max() < M)
    y = np.empty((nrows, H), dtype=np.float64)
    _load().oracle_ffn_rows(_p(xp), _dt(xp), ctypes.c_int64(M), ctypes.c_int64(H),
                            ctypes.c_int64(F), ctypes.c_int(E_local), _p(seg_offsets),
                            _p(W_gate), _p(W_up), _p(W_down), _dt(W_gate), _p(r),
                            ctypes.c_int64(nrows), _p(y))
    return y


def combine(y, K: int, slot_of_row, topk_w, tokens=None) -> np.ndarray:
    """fp64 out rows for `tokens` (all when None): sum_k w[n,k] * y[slot(n,k)]."""
    y = _c(y)
    M, H = y.shape
    N = M // K
    slot_of_row = _c(slot_of_row, np.int32)
    topk_w = _c(topk_w, np.float64)
    assert slot_of_row.size == N * K and topk_w.size == N * K
    if tokens is None:
        t, ntok = None, N
    else:
        t = _c(tokens, np.int64)
        ntok = t.size
    out = np.empty((ntok, H), dtype=np.float64)
    _load().oracle_combine(_p(y), _dt(y), ctypes.c_int64(N), ctypes.c_int64(H), ctypes.c_int(K),
                           _p(slot_of_row), _p(topk_w), _p(t), ctypes.c_int64(ntok), _p(out))
    return out


def logit_r64(x_row: np.ndarray, w_col: np.ndarray) -> np.float32:
    """One R64 dot product (used by the pins)."""
    x_row = _c(x_row)
    w = _c(w_col, np.float32).reshape(-1, 1)
    H = x_row.size
    return np.float32(_load().oracle_logit_r64(_p(x_row), _dt(x_row), ctypes.c_int64(H),
                                               ctypes.c_int64(0), _p(w), ctypes.c_int(1),
                                               ctypes.c_int(0)))
