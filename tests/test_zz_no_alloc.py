"""The entry point that allocates nothing (moe_dispatch_layout_static: histograms in an array built into
the library) against moe_dispatch_layout with a caller's workspace, through the C ABI: same bits, on two
calls in a row, the second with a smaller input that leaves the first call's histograms behind it."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _idx(rng, N, E, K, skew):
    p = None
    if skew:
        p = 1.0 / np.arange(1, E + 1) ** skew
        p /= p.sum()
    return np.stack([rng.choice(E, size=K, replace=False, p=p) for _ in range(N)]).astype(np.int32)


def _outputs(torch, E, G, R):
    i32 = dict(dtype=torch.int32, device="cuda:0")
    return [torch.full((n,), -7, **i32) for n in (E, E + 1, G, G + 1, R, R)]


def test_static_layout_equals_workspace_layout_on_two_calls_in_a_row():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import oracle
    import paper_2605_05888_amd as hub
    lib = hub.load_library(build_if_missing=False)
    rng = np.random.default_rng(2)
    stream = torch.cuda.current_stream().cuda_stream
    # (N, E, K, G, skew): a large skewed case, then a smaller one with other E and K, then an empty one
    for N, E, K, G, skew in [(9000, 256, 8, 32, 1.2), (700, 12, 3, 4, 0.0), (0, 8, 2, 2, 0.0), (3000, 64, 1, 8, 2.0)]:
        print("static layout", N, E, K, G, skew, flush=True)
        idx_h = _idx(rng, N, E, K, skew) if N else np.zeros((0, K), np.int32)
        idx = torch.from_numpy(idx_h).to("cuda:0")
        R = N * K
        want = _outputs(torch, E, G, R)
        ws_bytes = hub.workspace_bytes(hub.OP_DISPATCH_LAYOUT, N=N, E=E, K=K, G=G)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda:0")
        rc = lib.moe_dispatch_layout(idx.data_ptr(), N, K, E, G, *[t.data_ptr() for t in want], ws.data_ptr(),
                                     ws.numel(), stream)
        assert rc == 0, hub.last_error()
        got = _outputs(torch, E, G, R)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = lib.moe_dispatch_layout_static(idx.data_ptr(), N, K, E, G, *[t.data_ptr() for t in got], stream)
        assert rc == 0, hub.last_error()
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        o = oracle.layout(idx_h, E, G)
        names = ["expert_counts", "expert_offsets", "dest_counts", "dest_offsets", "slot_of_row", "row_of_slot"]
        for name, g, w in zip(names, got, want):
            assert torch.equal(g, w), name
            assert np.array_equal(g.cpu().numpy(), o[name]), name


def test_static_layout_rejects_sizes_beyond_its_array():
    import torch
    import paper_2605_05888_amd as hub
    lib = hub.load_library(build_if_missing=False)
    d = torch.zeros(16, dtype=torch.int32, device="cuda:0").data_ptr()
    N, K, E = 1 << 22, 2, 1024                      # 16384 units x 1024 experts x 4 bytes = 64 MiB
    assert hub.workspace_bytes(hub.OP_DISPATCH_LAYOUT, N=N, E=E, K=K, G=1) > (4 << 20)
    rc = lib.moe_dispatch_layout_static(d, N, K, E, 1, d, d, d, d, d, d, None)
    assert rc == -2 and "moe_dispatch_layout" in hub.last_error()
