"""The C-ABI library without a GPU: it loads, exports every declared symbol, and
rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2605_05888_amd as hub

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "moe_hub.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert set(names) == {"moe_last_error", "moe_workspace_bytes", "moe_route", "moe_dispatch_layout",
                          "moe_dispatch_layout_arrival", "moe_dispatch_layout_static", "moe_route_resolve_arrival",
                          "moe_permute", "moe_grouped_ffn", "moe_combine",
                          "moe_ffn_schedule", "moe_ffn_gate_up", "moe_ffn_gate_up_gather", "moe_ffn_down",
                          "moe_ffn_down_combine", "moe_ffn_status", "moe_ffn_gate_up_down"}
    lib = ctypes.CDLL(hub.lib_path()) if os.path.exists(hub.lib_path()) else hub.load_library()
    for n in names:
        assert hasattr(lib, n), n
    assert set(hub.exported_symbols()) == set(names)            # the binding covers the same set


def test_workspace_sizes():
    assert hub.workspace_bytes(hub.OP_ROUTE, N=100, E=8) == 100 * 8 * 4
    assert hub.workspace_bytes(hub.OP_DISPATCH_LAYOUT, N=16384, E=256, K=8) >= 256 * 256 * 4
    assert hub.workspace_bytes(hub.OP_DISPATCH_LAYOUT, N=0, E=8, K=2) == 0
    n = hub.workspace_bytes(hub.OP_GROUPED_FFN, N=8192, H=4096, E=8, F=14336, dtype=hub.BF16)
    assert n >= 8192 * 14336 * 2
    assert hub.workspace_bytes(hub.OP_GROUPED_FFN, N=512, H=128, E=8, F=256, dtype=hub.F32) >= 512 * 256 * 4
    assert hub.workspace_bytes(99) == 0


ALIGNED = 0x1000   # a fake, well-aligned, never-dereferenced pointer: every case below fails validation first


@pytest.mark.parametrize("call,code,word", [
    (lambda L: L.moe_permute(ALIGNED, 5, 4, 64, 2, ALIGNED, ALIGNED, ALIGNED, None), -2, "dtype"),
    (lambda L: L.moe_permute(ALIGNED, hub.BF16, 4, 60, 2, ALIGNED, ALIGNED, ALIGNED, None), -1, "16"),
    (lambda L: L.moe_permute(None, hub.BF16, 4, 64, 2, ALIGNED, ALIGNED, ALIGNED, None), -1, "NULL"),
    (lambda L: L.moe_permute(ALIGNED + 2, hub.BF16, 4, 64, 2, ALIGNED, ALIGNED, ALIGNED, None), -1, "aligned"),
    (lambda L: L.moe_permute(ALIGNED, hub.BF16, 1 << 30, 64, 4, ALIGNED, ALIGNED, ALIGNED, None), -1, "2^31"),
    (lambda L: L.moe_permute(ALIGNED, hub.BF16, 4, 64, 65, ALIGNED, ALIGNED, ALIGNED, None), -2, "K <= 64"),
    (lambda L: L.moe_ffn_status(hub.BF16, 100, 64, 64, 2, ALIGNED, 16, None), -3, "workspace"),
    (lambda L: L.moe_route(ALIGNED, hub.BF16, 4, 64, ALIGNED, None, 8, 9, 0, ALIGNED, ALIGNED, ALIGNED, None, 0, None),
     -1, "K"),
    (lambda L: L.moe_route(ALIGNED, hub.BF16, 4, 64, ALIGNED, None, 4096, 2, 0, ALIGNED, ALIGNED, ALIGNED, None, 0,
                           None), -2, "MOE_MAX_EXPERTS"),
    (lambda L: L.moe_route(ALIGNED, hub.BF16, 4, 64, ALIGNED, None, 8, 2, 3, ALIGNED, ALIGNED, ALIGNED, None, 0, None),
     -1, "score_mode"),
    (lambda L: L.moe_route(ALIGNED, hub.BF16, 4, 64, ALIGNED, None, 8, 2, 0, ALIGNED, ALIGNED, None, None, 0, None),
     -3, "workspace"),
    (lambda L: L.moe_dispatch_layout(ALIGNED, 4, 2, 8, 3, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED,
                                     ALIGNED, 1 << 20, None), -1, "divide"),
    (lambda L: L.moe_dispatch_layout(ALIGNED, 4, 2, 8, 2, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED,
                                     ALIGNED, 4, None), -3, "workspace"),
    (lambda L: L.moe_dispatch_layout(ALIGNED, 4, 2, 8, 2, None, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED,
                                     ALIGNED, 1 << 20, None), -1, "NULL"),
    (lambda L: L.moe_dispatch_layout_arrival(ALIGNED, 4, 2, 8, 3, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED,
                                             ALIGNED, None), -1, "divide"),
    (lambda L: L.moe_dispatch_layout_arrival(ALIGNED, 4, 2, 8, 2, ALIGNED, ALIGNED, ALIGNED, ALIGNED, None,
                                             ALIGNED, None), -1, "NULL"),
    (lambda L: L.moe_route_resolve_arrival(ALIGNED, hub.BF16, 4, 64, ALIGNED, None, 8, 2, 3, 0, ALIGNED, ALIGNED,
                                           ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED, None, 0, None),
     -1, "divide"),
    (lambda L: L.moe_route_resolve_arrival(ALIGNED, hub.BF16, 4, 64, ALIGNED, None, 8, 2, 2, 0, ALIGNED, ALIGNED,
                                           None, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED, None, 0, None),
     -3, "workspace"),
    (lambda L: L.moe_route_resolve_arrival(ALIGNED, hub.BF16, 4, 64, ALIGNED, None, 8, 2, 2, 0, ALIGNED, ALIGNED,
                                           ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED, None, ALIGNED, None, 0, None),
     -1, "NULL"),
    (lambda L: L.moe_grouped_ffn(ALIGNED, hub.BF16, 64, 64, 64, 0, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED,
                                 ALIGNED, 1 << 30, None), -1, "E_local"),
    (lambda L: L.moe_grouped_ffn(ALIGNED, hub.BF16, 64, 64, 64, 2, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED,
                                 None, 0, None), -3, "workspace"),
    (lambda L: L.moe_grouped_ffn(ALIGNED, hub.BF16, 64, 96, 64, 2, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED,
                                 ALIGNED, 1 << 30, None), -2, "multiples of 64"),
    (lambda L: L.moe_ffn_down_combine(hub.F32, 4, 2, 64, 64, 2, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED,
                                      ALIGNED, 1 << 30, None), -2, "BF16"),
    (lambda L: L.moe_ffn_down_combine(hub.BF16, 4, 0, 64, 64, 2, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED, ALIGNED,
                                      ALIGNED, 1 << 30, None), -1, "K"),
    (lambda L: L.moe_combine(ALIGNED, hub.BF16, 4, 64, 0, ALIGNED, ALIGNED, ALIGNED, None), -1, "K"),
    (lambda L: L.moe_combine(ALIGNED, hub.F32, 4, 6, 2, ALIGNED, ALIGNED, ALIGNED, None), -1, "16"),
])
def test_bad_arguments_are_rejected_before_any_launch(call, code, word):
    lib = hub.load_library()
    assert call(lib) == code
    assert word in hub.last_error()


def test_empty_inputs_are_successful_noops():
    lib = hub.load_library()
    assert lib.moe_permute(None, hub.BF16, 0, 64, 2, None, None, None, None) == 0
    assert lib.moe_combine(None, hub.BF16, 0, 64, 2, None, None, None, None) == 0
    assert lib.moe_route(None, hub.BF16, 0, 64, None, None, 8, 2, 0, None, None, None, None, 0, None) == 0
    assert lib.moe_grouped_ffn(None, hub.BF16, 0, 64, 64, 2, None, None, None, None, None, None, 0, None) == 0
    assert hub.last_error() == ""
