"""Test helper: allocates buffers with PyTorch and drives the C-ABI library step by step."""
from __future__ import annotations

import numpy as np
import torch

import moe_inputs as mi
import moe_inputs.device as mid
import paper_2605_05888_amd as hub

DEV = "cuda:0"


def tdtype(cfg):
    return torch.bfloat16 if cfg.dtype == mi.BF16 else torch.float32


def code(cfg):
    return hub.BF16 if cfg.dtype == mi.BF16 else hub.F32


def ws_tensor(nbytes: int):
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=DEV)


def gpu_route(x, W_r, bias, K, score_mode, want_logits=True):
    N, H = x.shape
    E = W_r.shape[1]
    idx = torch.full((N, K), -1, dtype=torch.int32, device=DEV)
    w = torch.zeros((N, K), dtype=torch.float32, device=DEV)
    logits = torch.zeros((N, E), dtype=torch.float32, device=DEV) if want_logits else None
    ws = None if want_logits else ws_tensor(hub.workspace_bytes(hub.OP_ROUTE, N=N, E=E))
    hub.moe_route(x, W_r, bias, K, score_mode, idx, w, logits, ws)
    return idx, w, logits


def gpu_layout(idx, E, G):
    N, K = idx.shape
    R = N * K
    out = dict(
        expert_counts=torch.full((E,), -7, dtype=torch.int32, device=DEV),
        expert_offsets=torch.full((E + 1,), -7, dtype=torch.int32, device=DEV),
        dest_counts=torch.full((G,), -7, dtype=torch.int32, device=DEV),
        dest_offsets=torch.full((G + 1,), -7, dtype=torch.int32, device=DEV),
        slot_of_row=torch.full((R,), -7, dtype=torch.int32, device=DEV),
        row_of_slot=torch.full((R,), -7, dtype=torch.int32, device=DEV))
    ws = ws_tensor(hub.workspace_bytes(hub.OP_DISPATCH_LAYOUT, N=N, E=E, K=K, G=G))
    hub.moe_dispatch_layout(idx, E, G, out["expert_counts"], out["expert_offsets"], out["dest_counts"],
                            out["dest_offsets"], out["slot_of_row"], out["row_of_slot"], ws)
    return out


def gpu_layout_arrival(idx, E, G):
    N, K = idx.shape
    R = N * K
    out = dict(
        expert_counts=torch.full((E,), -7, dtype=torch.int32, device=DEV),
        expert_offsets=torch.full((E + 1,), -7, dtype=torch.int32, device=DEV),
        dest_counts=torch.full((G,), -7, dtype=torch.int32, device=DEV),
        dest_offsets=torch.full((G + 1,), -7, dtype=torch.int32, device=DEV),
        slot_of_row=torch.full((R,), -7, dtype=torch.int32, device=DEV),
        row_of_slot=torch.full((R,), -7, dtype=torch.int32, device=DEV))
    hub.moe_dispatch_layout_arrival(idx, E, G, out["expert_counts"], out["expert_offsets"], out["dest_counts"],
                                    out["dest_offsets"], out["slot_of_row"], out["row_of_slot"])
    return out


def gpu_route_resolve_arrival(x, W_r, bias, K, G, score_mode):
    """Routing and arrival-order address resolution in one call: (idx, w, logits, layout dict)."""
    N, H = x.shape
    E = W_r.shape[1]
    R = N * K
    idx = torch.full((N, K), -1, dtype=torch.int32, device=DEV)
    w = torch.zeros((N, K), dtype=torch.float32, device=DEV)
    logits = torch.zeros((N, E), dtype=torch.float32, device=DEV)
    out = dict(
        expert_counts=torch.full((E,), -7, dtype=torch.int32, device=DEV),
        expert_offsets=torch.full((E + 1,), -7, dtype=torch.int32, device=DEV),
        dest_counts=torch.full((G,), -7, dtype=torch.int32, device=DEV),
        dest_offsets=torch.full((G + 1,), -7, dtype=torch.int32, device=DEV),
        slot_of_row=torch.full((R,), -7, dtype=torch.int32, device=DEV),
        row_of_slot=torch.full((R,), -7, dtype=torch.int32, device=DEV))
    hub.moe_route_resolve_arrival(x, W_r, bias, K, G, score_mode, idx, w, out["expert_counts"], out["expert_offsets"],
                                  out["dest_counts"], out["dest_offsets"], out["slot_of_row"], out["row_of_slot"],
                                  logits)
    return idx, w, logits, out


def gpu_permute(x, K, lay):
    N, H = x.shape
    xp = torch.zeros((N * K, H), dtype=x.dtype, device=DEV)
    hub.moe_permute(x, K, lay["slot_of_row"], lay["row_of_slot"], xp)
    return xp


def gpu_ffn(xp, seg_offsets, Wg, Wu, Wd):
    M, H = xp.shape
    E_local, F, _ = Wg.shape
    y = torch.zeros((M, H), dtype=xp.dtype, device=DEV)
    dt = hub.BF16 if xp.dtype == torch.bfloat16 else hub.F32
    ws = ws_tensor(hub.workspace_bytes(hub.OP_GROUPED_FFN, N=M, H=H, E=E_local, F=F, dtype=dt))
    hub.moe_grouped_ffn(xp, seg_offsets, Wg, Wu, Wd, y, ws)
    return y


def gpu_combine(y, K, slot_of_row, w):
    M, H = y.shape
    out = torch.zeros((M // K, H), dtype=y.dtype, device=DEV)
    hub.moe_combine(y, K, slot_of_row, w, out)
    return out


def host(t):
    return mid.to_host(t)


def as_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return mi.bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def check_close(got: np.ndarray, want: np.ndarray, max_abs: float, rel_l2: float, what: str = ""):
    """The floating-point bar: max-abs error and relative L2 error."""
    got = as_f64(got)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    err = np.abs(got - want)
    ma = float(err.max()) if err.size else 0.0
    den = float(np.linalg.norm(want.ravel()))
    rl = float(np.linalg.norm((got - want).ravel())) / den if den > 0 else 0.0
    assert ma <= max_abs, f"{what}: max-abs {ma:.3e} > {max_abs:.1e}"
    assert rl <= rel_l2, f"{what}: rel-L2 {rl:.3e} > {rel_l2:.1e}"
    return ma, rl


def tolerances(cfg):
    # bf16 storage with fp32 accumulation: max-abs 2e-2, rel-L2 1e-2; fp32: 1e-4 / 1e-5
    return (2e-2, 1e-2) if cfg.dtype == mi.BF16 else (1e-4, 1e-5)
