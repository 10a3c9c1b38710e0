"""ctypes binding of ``include/moe_hub.h``: same names, argument marshalling only."""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
# MOE_HUB_LIBRARY selects another build of the same library (A/B timing of two builds)
_LIB_PATH = os.environ.get("MOE_HUB_LIBRARY") or os.path.join(HERE, "libmoe_hub.so")

BF16, F32 = 0, 1
SCORE_SOFTMAX_TOPK, SCORE_SIGMOID_TOPK = 0, 1
OP_ROUTE, OP_DISPATCH_LAYOUT, OP_GROUPED_FFN = 0, 1, 2

_ERR_NAMES = {-1: "MOE_ERR_ARG", -2: "MOE_ERR_UNSUPPORTED", -3: "MOE_ERR_WORKSPACE", -4: "MOE_ERR_LAUNCH",
              -5: "MOE_ERR_STATE"}

_c_i64, _c_int, _c_vp, _c_sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t

# name -> (restype, argtypes), exactly the declarations of include/moe_hub.h
_SIGNATURES = {
    "moe_last_error": (ctypes.c_char_p, []),
    "moe_workspace_bytes": (_c_sz, [_c_int, _c_i64, _c_i64, _c_int, _c_int, _c_int, _c_i64, _c_int]),
    "moe_route": (_c_int, [_c_vp, _c_int, _c_i64, _c_i64, _c_vp, _c_vp, _c_int, _c_int, _c_int,
                           _c_vp, _c_vp, _c_vp, _c_vp, _c_sz, _c_vp]),
    "moe_dispatch_layout": (_c_int, [_c_vp, _c_i64, _c_int, _c_int, _c_int, _c_vp, _c_vp, _c_vp, _c_vp,
                                     _c_vp, _c_vp, _c_vp, _c_sz, _c_vp]),
    "moe_dispatch_layout_static": (_c_int, [_c_vp, _c_i64, _c_int, _c_int, _c_int, _c_vp, _c_vp, _c_vp,
                                            _c_vp, _c_vp, _c_vp, _c_vp]),
    "moe_dispatch_layout_arrival": (_c_int, [_c_vp, _c_i64, _c_int, _c_int, _c_int, _c_vp, _c_vp, _c_vp,
                                             _c_vp, _c_vp, _c_vp, _c_vp]),
    "moe_route_resolve_arrival": (_c_int, [_c_vp, _c_int, _c_i64, _c_i64, _c_vp, _c_vp, _c_int, _c_int, _c_int,
                                           _c_int, _c_vp, _c_vp, _c_vp, _c_vp, _c_vp, _c_vp, _c_vp, _c_vp, _c_vp,
                                           _c_vp, _c_sz, _c_vp]),
    "moe_permute": (_c_int, [_c_vp, _c_int, _c_i64, _c_i64, _c_int, _c_vp, _c_vp, _c_vp, _c_vp]),
    "moe_grouped_ffn": (_c_int, [_c_vp, _c_int, _c_i64, _c_i64, _c_i64, _c_int, _c_vp, _c_vp, _c_vp,
                                 _c_vp, _c_vp, _c_vp, _c_sz, _c_vp]),
    "moe_ffn_schedule": (_c_int, [_c_int, _c_i64, _c_i64, _c_i64, _c_int, _c_vp, _c_vp, _c_sz, _c_vp]),
    "moe_ffn_gate_up_down": (_c_int, [_c_vp, _c_int, _c_i64, _c_i64, _c_i64, _c_int, _c_vp, _c_vp, _c_vp,
                                      _c_vp, _c_vp, _c_vp, _c_sz, _c_i64, _c_vp]),
    "moe_ffn_status": (_c_int, [_c_int, _c_i64, _c_i64, _c_i64, _c_int, _c_vp, _c_sz, _c_vp]),
    "moe_ffn_gate_up": (_c_int, [_c_vp, _c_int, _c_i64, _c_i64, _c_i64, _c_int, _c_vp, _c_vp, _c_vp,
                                 _c_vp, _c_sz, _c_vp]),
    "moe_ffn_gate_up_gather": (_c_int, [_c_vp, _c_int, _c_i64, _c_int, _c_i64, _c_i64, _c_int, _c_vp, _c_vp,
                                        _c_vp, _c_vp, _c_vp, _c_sz, _c_vp]),
    "moe_ffn_down_combine": (_c_int, [_c_int, _c_i64, _c_int, _c_i64, _c_i64, _c_int, _c_vp, _c_vp, _c_vp, _c_vp,
                                      _c_vp, _c_vp, _c_vp, _c_sz, _c_vp]),
    "moe_ffn_down": (_c_int, [_c_int, _c_i64, _c_i64, _c_i64, _c_int, _c_vp, _c_vp, _c_vp, _c_vp, _c_sz, _c_vp]),
    "moe_combine": (_c_int, [_c_vp, _c_int, _c_i64, _c_i64, _c_int, _c_vp, _c_vp, _c_vp, _c_vp]),
}

_lib = None


class MoEHubError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"{_ERR_NAMES.get(code, code)}: {message}")
        self.code = code


def lib_path() -> str:
    return _LIB_PATH


def exported_symbols():
    return sorted(_SIGNATURES)


def load_library(build_if_missing: bool = True):
    """Loads libmoe_hub.so (building it with hipcc when it does not exist yet)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(f"{_LIB_PATH} is not built; run python -m paper_2605_05888_amd.build")
        from . import build as _build
        _build.build(verbose=False)
    lib = ctypes.CDLL(_LIB_PATH)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)          # AttributeError if a declared symbol is missing
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def last_error() -> str:
    return load_library().moe_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise MoEHubError(rc, last_error())


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported activation dtype {t.dtype}")


def _need(t, dtype, name):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise TypeError(f"{name} must be a contiguous device tensor of {dtype}")


def workspace_bytes(op: int, N: int = 0, H: int = 0, E: int = 0, K: int = 0, G: int = 1, F: int = 0,
                    dtype: int = BF16) -> int:
    return int(load_library().moe_workspace_bytes(op, N, H, E, K, G, F, dtype))


def _ws_args(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def moe_route(x, W_r, bias, K: int, score_mode: int, topk_idx, topk_w, logits=None, ws=None):
    import torch
    N, H = x.shape
    E = W_r.shape[1]
    _need(W_r, torch.float32, "W_r")
    _need(topk_idx, torch.int32, "topk_idx")
    _need(topk_w, torch.float32, "topk_w")
    assert W_r.shape[0] == H and x.is_contiguous()
    assert topk_idx.numel() == N * K and topk_w.numel() == N * K
    assert logits is None or (logits.numel() == N * E and logits.dtype == torch.float32)
    wp, wb = _ws_args(ws)
    _check(load_library().moe_route(_ptr(x), _dtype_code(x), N, H, _ptr(W_r), _ptr(bias), E, K, score_mode,
                                    _ptr(topk_idx), _ptr(topk_w), _ptr(logits), wp, wb, _stream()))


def moe_dispatch_layout(topk_idx, E: int, G: int, expert_counts, expert_offsets, dest_counts, dest_offsets,
                        slot_of_row, row_of_slot, ws):
    import torch
    N, K = topk_idx.shape
    for name, t, n in (("expert_counts", expert_counts, E), ("expert_offsets", expert_offsets, E + 1),
                       ("dest_counts", dest_counts, G), ("dest_offsets", dest_offsets, G + 1),
                       ("slot_of_row", slot_of_row, N * K), ("row_of_slot", row_of_slot, N * K)):
        _need(t, torch.int32, name)
        assert t.numel() == n, name
    _need(topk_idx, torch.int32, "topk_idx")
    wp, wb = _ws_args(ws)
    _check(load_library().moe_dispatch_layout(_ptr(topk_idx), N, K, E, G, _ptr(expert_counts),
                                              _ptr(expert_offsets), _ptr(dest_counts), _ptr(dest_offsets),
                                              _ptr(slot_of_row), _ptr(row_of_slot), wp, wb, _stream()))


def moe_dispatch_layout_static(topk_idx, E: int, G: int, expert_counts, expert_offsets, dest_counts,
                               dest_offsets, slot_of_row, row_of_slot):
    import torch
    N, K = topk_idx.shape
    for name, t, n in (("expert_counts", expert_counts, E), ("expert_offsets", expert_offsets, E + 1),
                       ("dest_counts", dest_counts, G), ("dest_offsets", dest_offsets, G + 1),
                       ("slot_of_row", slot_of_row, N * K), ("row_of_slot", row_of_slot, N * K)):
        _need(t, torch.int32, name)
        assert t.numel() == n, name
    _need(topk_idx, torch.int32, "topk_idx")
    _check(load_library().moe_dispatch_layout_static(_ptr(topk_idx), N, K, E, G, _ptr(expert_counts),
                                                     _ptr(expert_offsets), _ptr(dest_counts),
                                                     _ptr(dest_offsets), _ptr(slot_of_row),
                                                     _ptr(row_of_slot), _stream()))


def moe_dispatch_layout_arrival(topk_idx, E: int, G: int, expert_counts, expert_offsets, dest_counts,
                                dest_offsets, slot_of_row, row_of_slot):
    import torch
    N, K = topk_idx.shape
    for name, t, n in (("expert_counts", expert_counts, E), ("expert_offsets", expert_offsets, E + 1),
                       ("dest_counts", dest_counts, G), ("dest_offsets", dest_offsets, G + 1),
                       ("slot_of_row", slot_of_row, N * K), ("row_of_slot", row_of_slot, N * K)):
        _need(t, torch.int32, name)
        assert t.numel() == n, name
    _need(topk_idx, torch.int32, "topk_idx")
    _check(load_library().moe_dispatch_layout_arrival(_ptr(topk_idx), N, K, E, G, _ptr(expert_counts),
                                                      _ptr(expert_offsets), _ptr(dest_counts),
                                                      _ptr(dest_offsets), _ptr(slot_of_row),
                                                      _ptr(row_of_slot), _stream()))


def moe_route_resolve_arrival(x, W_r, bias, K: int, G: int, score_mode: int, topk_idx, topk_w, expert_counts,
                              expert_offsets, dest_counts, dest_offsets, slot_of_row, row_of_slot, logits=None,
                              ws=None):
    import torch
    N, H = x.shape
    E = W_r.shape[1]
    _need(W_r, torch.float32, "W_r")
    _need(topk_idx, torch.int32, "topk_idx")
    _need(topk_w, torch.float32, "topk_w")
    assert W_r.shape[0] == H and x.is_contiguous()
    assert topk_idx.numel() == N * K and topk_w.numel() == N * K
    assert logits is None or (logits.numel() == N * E and logits.dtype == torch.float32)
    for name, t, n in (("expert_counts", expert_counts, E), ("expert_offsets", expert_offsets, E + 1),
                       ("dest_counts", dest_counts, G), ("dest_offsets", dest_offsets, G + 1),
                       ("slot_of_row", slot_of_row, N * K), ("row_of_slot", row_of_slot, N * K)):
        _need(t, torch.int32, name)
        assert t.numel() == n, name
    wp, wb = _ws_args(ws)
    _check(load_library().moe_route_resolve_arrival(
        _ptr(x), _dtype_code(x), N, H, _ptr(W_r), _ptr(bias), E, K, G, score_mode, _ptr(topk_idx), _ptr(topk_w),
        _ptr(logits), _ptr(expert_counts), _ptr(expert_offsets), _ptr(dest_counts), _ptr(dest_offsets),
        _ptr(slot_of_row), _ptr(row_of_slot), wp, wb, _stream()))


def moe_permute(x, K: int, slot_of_row, row_of_slot, xp):
    N, H = x.shape
    assert x.is_contiguous() and xp.is_contiguous() and xp.dtype == x.dtype and xp.numel() == N * K * H
    assert slot_of_row.numel() == N * K and row_of_slot.numel() == N * K
    _check(load_library().moe_permute(_ptr(x), _dtype_code(x), N, H, K, _ptr(slot_of_row), _ptr(row_of_slot),
                                      _ptr(xp), _stream()))


def moe_grouped_ffn(xp, seg_offsets, W_gate, W_up, W_down, y, ws):
    import torch
    M, H = xp.shape
    E_local, F, H2 = W_gate.shape
    assert H2 == H and tuple(W_up.shape) == (E_local, F, H) and tuple(W_down.shape) == (E_local, H, F)
    assert W_gate.dtype == W_up.dtype == W_down.dtype == xp.dtype == y.dtype
    for t in (xp, W_gate, W_up, W_down, y):
        assert t.is_cuda and t.is_contiguous()
    _need(seg_offsets, torch.int32, "seg_offsets")
    assert seg_offsets.numel() == E_local + 1 and y.numel() == M * H
    wp, wb = _ws_args(ws)
    _check(load_library().moe_grouped_ffn(_ptr(xp), _dtype_code(xp), M, H, F, E_local, _ptr(seg_offsets),
                                          _ptr(W_gate), _ptr(W_up), _ptr(W_down), _ptr(y), wp, wb, _stream()))


def moe_ffn_schedule(dtype: int, M: int, H: int, F: int, seg_offsets, ws):
    wp, wb = _ws_args(ws)
    _check(load_library().moe_ffn_schedule(dtype, M, H, F, seg_offsets.numel() - 1, _ptr(seg_offsets), wp, wb,
                                           _stream()))


def moe_ffn_gate_up_down(xp, seg_offsets, W_gate, W_up, W_down, y, ws, wait_limit: int = 0):
    import torch
    M, H = xp.shape
    E_local, F, H2 = W_gate.shape
    assert H2 == H and tuple(W_up.shape) == (E_local, F, H) and tuple(W_down.shape) == (E_local, H, F)
    assert W_gate.dtype == W_up.dtype == W_down.dtype == xp.dtype == y.dtype
    for t in (xp, W_gate, W_up, W_down, y):
        assert t.is_cuda and t.is_contiguous()
    _need(seg_offsets, torch.int32, "seg_offsets")
    assert seg_offsets.numel() == E_local + 1 and y.numel() == M * H
    wp, wb = _ws_args(ws)
    _check(load_library().moe_ffn_gate_up_down(_ptr(xp), _dtype_code(xp), M, H, F, E_local, _ptr(seg_offsets),
                                               _ptr(W_gate), _ptr(W_up), _ptr(W_down), _ptr(y), wp, wb,
                                               wait_limit, _stream()))


def moe_ffn_status(dtype: int, M: int, H: int, F: int, E_local: int, ws):
    """Waits for the current stream; raises MoEHubError(MOE_ERR_STATE) if a GEMM step found no schedule."""
    wp, wb = _ws_args(ws)
    _check(load_library().moe_ffn_status(dtype, M, H, F, E_local, wp, wb, _stream()))


def moe_ffn_gate_up(xp, seg_offsets, W_gate, W_up, ws):
    M, H = xp.shape
    E_local, F, _ = W_gate.shape
    assert tuple(W_up.shape) == tuple(W_gate.shape) and W_gate.shape[2] == H
    assert xp.is_contiguous() and W_gate.is_contiguous() and W_up.is_contiguous()
    assert seg_offsets.numel() == E_local + 1
    wp, wb = _ws_args(ws)
    _check(load_library().moe_ffn_gate_up(_ptr(xp), _dtype_code(xp), M, H, F, E_local, _ptr(seg_offsets),
                                          _ptr(W_gate), _ptr(W_up), wp, wb, _stream()))


def moe_ffn_gate_up_gather(x, K: int, seg_offsets, row_of_slot, W_gate, W_up, ws):
    import torch
    N, H = x.shape
    E_local, F, _ = W_gate.shape
    assert tuple(W_up.shape) == tuple(W_gate.shape) and W_gate.shape[2] == H
    assert x.is_contiguous() and W_gate.is_contiguous() and W_up.is_contiguous()
    assert seg_offsets.numel() == E_local + 1
    _need(row_of_slot, torch.int32, "row_of_slot")
    assert row_of_slot.numel() == N * K
    wp, wb = _ws_args(ws)
    _check(load_library().moe_ffn_gate_up_gather(_ptr(x), _dtype_code(x), N, K, H, F, E_local, _ptr(seg_offsets),
                                                 _ptr(row_of_slot), _ptr(W_gate), _ptr(W_up), wp, wb, _stream()))


def moe_ffn_down(seg_offsets, W_down, y, ws):
    M, H = y.shape
    E_local, H2, F = W_down.shape
    assert H2 == H and y.is_contiguous() and W_down.is_contiguous() and W_down.dtype == y.dtype
    assert seg_offsets.numel() == E_local + 1
    wp, wb = _ws_args(ws)
    _check(load_library().moe_ffn_down(_dtype_code(y), M, H, F, E_local, _ptr(seg_offsets), _ptr(W_down),
                                       _ptr(y), wp, wb, _stream()))


def moe_ffn_down_combine(K: int, seg_offsets, W_down, row_of_slot, topk_w, sums, out, ws):
    import torch
    N, H = out.shape
    E_local, H2, F = W_down.shape
    assert H2 == H and out.is_contiguous() and W_down.is_contiguous() and W_down.dtype == out.dtype
    assert seg_offsets.numel() == E_local + 1
    _need(row_of_slot, torch.int32, "row_of_slot")
    _need(topk_w, torch.float32, "topk_w")
    _need(sums, torch.float32, "sums")
    assert row_of_slot.numel() == N * K and topk_w.numel() == N * K and sums.numel() == N * H
    wp, wb = _ws_args(ws)
    _check(load_library().moe_ffn_down_combine(_dtype_code(out), N, K, H, F, E_local, _ptr(seg_offsets),
                                               _ptr(W_down), _ptr(row_of_slot), _ptr(topk_w), _ptr(sums),
                                               _ptr(out), wp, wb, _stream()))


def moe_combine(y, K: int, slot_of_row, topk_w, out):
    import torch
    N, H = out.shape
    assert y.is_contiguous() and out.is_contiguous() and y.dtype == out.dtype and y.numel() == N * K * H
    _need(topk_w, torch.float32, "topk_w")
    assert slot_of_row.numel() == N * K and topk_w.numel() == N * K
    _check(load_library().moe_combine(_ptr(y), _dtype_code(y), N, H, K, _ptr(slot_of_row), _ptr(topk_w),
                                      _ptr(out), _stream()))
