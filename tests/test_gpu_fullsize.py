"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Routing, layout and permutation are compared in full (bit-exact).  The expert FFN is
compared on 500+ sampled rows the oracle computes one by one, chosen deterministically:
first and last row of every non-empty expert segment, one row in every 32-row block of a few
tiles of every kind the workload has (full, tall, ragged, shallow), evenly spaced rows, and
every slot of a few sampled tokens so that the layer output of those tokens is checked end to
end.  The combine step is compared in full: every token, against the oracle's combine of the
GPU's own y.  Inputs are generated in
HBM by the harness fill kernel (identical, bit for bit, to the host generator) and copied
back for the oracle; nothing the oracle consumes comes from the library under test.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import moe_inputs as mi  # noqa: E402
import oracle  # noqa: E402

FULL = ["mixtral", "gptoss", "dsv3", "dsv3_ep", "qwen2moe", "phi35moe"]
_state = {}


def _say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import gpu_layer
    import paper_2605_05888_amd as hub
    hub.load_library(build_if_missing=False)
    return gpu_layer


def _get(G, name):
    """Device inputs and the GPU's routing/layout/permute outputs for one workload (cached)."""
    import torch
    import moe_inputs.device as mid
    if _state.get("name") == name:
        return _state
    _state.clear()
    torch.cuda.empty_cache()
    cfg = mi.CONFIGS[name]
    _say("setting up", cfg)
    s = _state
    s["name"], s["cfg"] = name, cfg
    s["x"] = mid.device_tensor(cfg, mi.STREAM_X)
    s["W_r"] = mid.device_tensor(cfg, mi.STREAM_W_ROUTER)
    bias = mi.router_bias(cfg)
    s["bias_h"] = bias
    s["bias"] = None if bias is None else mid.to_device(bias)
    s["E_local"] = cfg.E // cfg.G
    s["W"] = tuple(mid.device_tensor(cfg, st, 0, s["E_local"])
                   for st in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    s["idx"], s["w"], _ = G.gpu_route(s["x"], s["W_r"], s["bias"], cfg.K, cfg.score_mode, want_logits=False)
    s["lay"] = G.gpu_layout(s["idx"], cfg.E, cfg.G)
    s["xp"] = G.gpu_permute(s["x"], cfg.K, s["lay"])
    torch.cuda.synchronize()
    return s


def _oracle_routing(G, s):
    if "o_idx" not in s:
        cfg = s["cfg"]
        s["x_h"] = G.host(s["x"])
        s["o_idx"], s["o_w"], _ = oracle.route(s["x_h"], G.host(s["W_r"]), s["bias_h"], cfg.K, cfg.score_mode)
        s["o_lay"] = oracle.layout(s["o_idx"], cfg.E, cfg.G)
    return s


@pytest.fixture(scope="module", params=FULL)
def S(request, G):
    """Module-scoped and parametrised: pytest runs all tests of one workload before the next."""
    return _get(G, request.param)


def test_full_routing_and_layout_bit_exact(G, S):
    s = _oracle_routing(G, S)
    name = s["name"]
    cfg = s["cfg"]
    assert np.array_equal(G.host(s["idx"]), s["o_idx"])
    assert np.max(np.abs(G.host(s["w"]).astype(np.float64) - s["o_w"])) <= 2e-6
    for k, v in s["o_lay"].items():
        assert np.array_equal(G.host(s["lay"][k]), v), k
    cnt = s["o_lay"]["expert_counts"]
    share = cnt / cnt.sum()
    _say(f"   {name}: rows/expert min {cnt.min()} mean {cnt.mean():.0f} max {cnt.max()}; "
         f"std of per-expert token share {share.std():.4f}")


def test_full_permute_bitwise(G, S):
    s = _oracle_routing(G, S)
    cfg = s["cfg"]
    want = oracle.permute(s["x_h"], cfg.K, s["o_lay"]["slot_of_row"])
    assert np.array_equal(G.host(s["xp"]), want)
    s["o_xp"] = want


def _sample_rows(rng, seg, per_expert):
    rows = []
    for e in range(len(seg) - 1):
        lo, hi = int(seg[e]), int(seg[e + 1])
        if hi > lo:
            rows += [lo, hi - 1]
            rows += list(rng.integers(lo, hi, size=per_expert))
    return np.unique(np.array(rows, dtype=np.int64))


# what the grouped GEMM makes of an expert with `rows` rows (csrc/ffn.hip): at most 64 rows: one shallow
# tile; otherwise tiles of 256 rows, a remainder of up to 64 rows riding with the last full tile ("tall"),
# a longer remainder forming a ragged tile of its own
TILE_ROWS, TALL_EXTRA, SHALLOW_ROWS = 256, 64, 64


def _tiles_of(lo, hi):
    """(kind, first row, rows) for every tile of the expert segment [lo, hi)."""
    n = hi - lo
    if n == 0:
        return []
    if n <= SHALLOW_ROWS:
        return [("shallow", lo, n)]
    full, rest = divmod(n, TILE_ROWS)
    tiles = [("full", lo + i * TILE_ROWS, TILE_ROWS) for i in range(full)]
    if full > 0 and 0 < rest <= TALL_EXTRA:
        tiles[-1] = ("tall", lo + (full - 1) * TILE_ROWS, TILE_ROWS + rest)
    elif rest > 0:
        tiles.append(("ragged", lo + full * TILE_ROWS, rest))
    return tiles


def _block_sweep(first, rows):
    """One row in every 32-row block of a tile, at a position inside the block that moves from block to block."""
    out = []
    for blk in range((rows + 31) // 32):
        out.append(first + min(blk * 32 + (blk * 7 + 3) % 32, rows - 1))
    return out


def _deterministic_sample(seg, want=560, tiles_per_kind=3):
    """First and last row of every expert; one row in every 32-row block of `tiles_per_kind` tiles of every
    kind the workload has (full, tall, ragged, shallow), taken from experts spread over the range; then
    evenly spaced rows until there are `want` of them."""
    lo_all, hi_all = int(seg[0]), int(seg[-1])
    rows, by_kind = [], {}
    for e in range(len(seg) - 1):
        lo, hi = int(seg[e]), int(seg[e + 1])
        if hi > lo:
            rows += [lo, hi - 1]
        for t in _tiles_of(lo, hi):
            by_kind.setdefault(t[0], []).append(t)
    kinds = {}
    for kind, tiles in by_kind.items():
        pick = [tiles[i * (len(tiles) - 1) // max(tiles_per_kind - 1, 1)] for i in range(min(tiles_per_kind, len(tiles)))]
        kinds[kind] = len(tiles)
        for _, first, n in pick:
            rows += _block_sweep(first, n)
    rows = np.unique(np.array(rows, dtype=np.int64))
    if rows.size < want and hi_all > lo_all:
        fill = np.linspace(lo_all, hi_all - 1, want - rows.size + 2).astype(np.int64)
        rows = np.unique(np.concatenate([rows, fill]))
    return rows, kinds


def _oracle_rows_by_expert(G, xp_h, seg, W_dev, rows):
    """Oracle FFN of `rows`, expert by expert (weights copied back one expert at a time)."""
    out = np.zeros((rows.size, xp_h.shape[1]), dtype=np.float64)
    e_of = np.searchsorted(np.asarray(seg[1:]), rows, side="right")
    for e in np.unique(e_of):
        sel = np.nonzero(e_of == e)[0]
        Wg, Wu, Wd = (G.host(w[e:e + 1]) for w in W_dev)
        out[sel] = oracle.ffn_rows(xp_h, np.array([seg[e], seg[e + 1]], np.int32), Wg, Wu, Wd, rows=rows[sel])
    return out


def test_full_ffn_on_samples_and_combine_in_full(G, S):
    import torch
    s = _oracle_routing(G, S)
    name = s["name"]
    cfg = s["cfg"]
    if "o_xp" not in s:
        s["o_xp"] = oracle.permute(s["x_h"], cfg.K, s["o_lay"]["slot_of_row"])
    o_lay, xp_h = s["o_lay"], s["o_xp"]
    El = s["E_local"]
    seg_h = o_lay["expert_offsets"][:El + 1]                 # destination 0's experts (all experts when G = 1)
    seg_d = s["lay"]["expert_offsets"][:El + 1].contiguous()
    lo, hi = int(seg_h[0]), int(seg_h[-1])
    # GPU: rows of other destinations keep the identity-expert value y = xp
    y = s["xp"].clone()
    M, H = y.shape
    import paper_2605_05888_amd as hub
    ws = G.ws_tensor(hub.workspace_bytes(hub.OP_GROUPED_FFN, N=M, H=H, E=El, F=cfg.F, dtype=hub.BF16))
    hub.moe_grouped_ffn(s["xp"], seg_d, *s["W"], y, ws)
    out = G.gpu_combine(y, cfg.K, s["lay"]["slot_of_row"], s["w"])
    torch.cuda.synchronize()
    rng = np.random.default_rng(cfg.seed + 100)
    tokens = rng.choice(cfg.N, size=8, replace=False)
    tok_slots = o_lay["slot_of_row"].reshape(cfg.N, cfg.K)[tokens].ravel().astype(np.int64)
    local = (tok_slots >= lo) & (tok_slots < hi)
    sample, kinds = _deterministic_sample(seg_h)
    rows = np.unique(np.concatenate([sample, tok_slots[local]]))
    _say(f"   {name}: oracle FFN on {rows.size} sampled rows of {hi - lo}; tiles by kind {kinds}")
    assert rows.size >= min(500, hi - lo)
    want = _oracle_rows_by_expert(G, xp_h, seg_h, s["W"], rows)
    y_h = G.host(y[torch.from_numpy(rows).to(y.device)])
    ma, rl = G.check_close(y_h, want, 2e-2, 1e-2, what="ffn rows")
    _say(f"   ffn max-abs {ma:.3e} rel-L2 {rl:.3e}")
    if lo > 0 or hi < M:                                      # rows of other destinations untouched
        probe = np.array([r for r in (0, lo - 1, hi, M - 1) if (0 <= r < lo or hi <= r < M)], dtype=np.int64)
        assert np.array_equal(G.host(y[torch.from_numpy(probe).to(y.device)]), xp_h[probe])
    # layer output of the sampled tokens: oracle FFN rows where local, identity elsewhere
    pos = {int(r): i for i, r in enumerate(rows)}
    y_c = np.stack([want[pos[int(r)]] if l else G.as_f64(xp_h[r]) for r, l in zip(tok_slots, local)])
    o_out = oracle.combine(y_c, cfg.K, np.arange(tok_slots.size, dtype=np.int32), s["o_w"][tokens])
    got = G.host(out[torch.from_numpy(tokens).to(out.device)])
    ma, rl = G.check_close(got, o_out, 2e-2, 1e-2, what="layer output")
    _say(f"   out max-abs {ma:.3e} rel-L2 {rl:.3e}")
    # the combine step in full: every token of `out` against the oracle's combine of the GPU's own y
    y_all = G.host(y)
    del y
    o_all = oracle.combine(y_all, cfg.K, o_lay["slot_of_row"], s["o_w"])
    ma, rl = G.check_close(G.host(out), o_all, 2e-2, 4e-3, what="combine, all tokens")
    _say(f"   combine over all {cfg.N} tokens: max-abs {ma:.3e} rel-L2 {rl:.3e}")


@pytest.mark.parametrize("N", [128, 512])
def test_mixtral_shape_at_small_token_counts(G, N):
    """The small end of the token-count sweep, at the full Mixtral H and F: every expert has a few dozen
    rows (N = 128: shallow tiles only) or one ragged tile (N = 512).  Routing, layout and permutation in
    full; the FFN on sampled rows; the layer output of the tokens whose rows were all sampled."""
    import dataclasses
    import torch
    import moe_inputs.device as mid
    import paper_2605_05888_amd as hub
    _state.clear()
    torch.cuda.empty_cache()
    cfg = dataclasses.replace(mi.CONFIGS["mixtral"], N=N)
    _say("mixtral shape,", N, "tokens")
    x = mid.device_tensor(cfg, mi.STREAM_X)
    W_r = mid.device_tensor(cfg, mi.STREAM_W_ROUTER)
    W = tuple(mid.device_tensor(cfg, st) for st in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    idx, w, _ = G.gpu_route(x, W_r, None, cfg.K, cfg.score_mode, want_logits=False)
    lay = G.gpu_layout(idx, cfg.E, cfg.G)
    xp = G.gpu_permute(x, cfg.K, lay)
    y = G.gpu_ffn(xp, lay["expert_offsets"], *W)
    out = G.gpu_combine(y, cfg.K, lay["slot_of_row"], w)
    torch.cuda.synchronize()
    x_h = G.host(x)
    o_idx, o_w, _ = oracle.route(x_h, G.host(W_r), None, cfg.K, cfg.score_mode)
    o_lay = oracle.layout(o_idx, cfg.E, cfg.G)
    o_xp = oracle.permute(x_h, cfg.K, o_lay["slot_of_row"])
    assert np.array_equal(G.host(idx), o_idx)
    for k, v in o_lay.items():
        assert np.array_equal(G.host(lay[k]), v), k
    assert np.array_equal(G.host(xp), o_xp)
    seg = o_lay["expert_offsets"]
    tokens = np.arange(0, N, max(1, N // 24))[:24]
    tok_slots = o_lay["slot_of_row"].reshape(N, cfg.K)[tokens].ravel().astype(np.int64)
    sample, kinds = _deterministic_sample(seg, want=96, tiles_per_kind=2)
    rows = np.unique(np.concatenate([sample, tok_slots]))
    _say(f"   rows per expert {np.diff(seg).tolist()}; tiles by kind {kinds}; {rows.size} sampled rows")
    want = _oracle_rows_by_expert(G, o_xp, seg, W, rows)
    ma, rl = G.check_close(G.host(y)[rows], want, 2e-2, 1e-2, what="ffn rows")
    _say(f"   ffn max-abs {ma:.3e} rel-L2 {rl:.3e}")
    pos = {int(r): i for i, r in enumerate(rows)}
    y_c = np.stack([want[pos[int(r)]] for r in tok_slots])
    o_out = oracle.combine(y_c, cfg.K, np.arange(tok_slots.size, dtype=np.int32), o_w[tokens])
    ma, rl = G.check_close(G.host(out)[tokens], o_out, 2e-2, 1e-2, what="layer output")
    _say(f"   out max-abs {ma:.3e} rel-L2 {rl:.3e}")
    o_all = oracle.combine(G.host(y), cfg.K, o_lay["slot_of_row"], o_w)
    G.check_close(G.host(out), o_all, 2e-2, 4e-3, what="combine, all tokens")


def test_full_ffn_in_one_launch_equals_two_launches(G, S):
    """At full size, in the configuration bench.py times: moe_ffn_gate_up_down (a down-projection tile starts
    when its rows have arrived) gives the y of moe_ffn_gate_up + moe_ffn_down, bit for bit, on two launches
    over one schedule."""
    import torch
    import paper_2605_05888_amd as hub
    s = S
    cfg = s["cfg"]
    El = s["E_local"]
    M, H = s["xp"].shape
    seg = s["lay"]["expert_offsets"][:El + 1].contiguous()
    ws = G.ws_tensor(hub.workspace_bytes(hub.OP_GROUPED_FFN, N=M, H=H, E=El, F=cfg.F, dtype=hub.BF16))
    hub.moe_ffn_schedule(hub.BF16, M, H, cfg.F, seg, ws)
    y0 = torch.zeros((M, H), dtype=torch.bfloat16, device="cuda:0")
    hub.moe_ffn_gate_up(s["xp"], seg, s["W"][0], s["W"][1], ws)
    hub.moe_ffn_down(seg, s["W"][2], y0, ws)
    for _ in range(2):
        y = torch.zeros((M, H), dtype=torch.bfloat16, device="cuda:0")
        ws[:M * cfg.F * 2].zero_()
        hub.moe_ffn_gate_up_down(s["xp"], seg, *s["W"], y, ws)
        hub.moe_ffn_status(hub.BF16, M, H, cfg.F, El, ws)
        assert torch.equal(y, y0)
        del y
    assert bool(y0.any())


def test_full_gate_up_with_fused_gather_is_bit_identical(G, S):
    """At full size: GEMM1 fetching its rows from x through row_of_slot leaves the same activation in
    the workspace as GEMM1 over the materialised xp (whose sampled rows the test above checks)."""
    import torch
    import paper_2605_05888_amd as hub
    s = S
    cfg = s["cfg"]
    if cfg.G != 1:
        pytest.skip("an expert-parallel rank computes received rows, not its own")
    M, H = s["xp"].shape
    seg = s["lay"]["expert_offsets"]
    nb = hub.workspace_bytes(hub.OP_GROUPED_FFN, N=M, H=H, E=cfg.E, F=cfg.F, dtype=hub.BF16)
    a_bytes = M * cfg.F * 2
    got = []
    for fused in (False, True):
        ws = G.ws_tensor(nb)
        hub.moe_ffn_schedule(hub.BF16, M, H, cfg.F, seg, ws)
        if fused:
            hub.moe_ffn_gate_up_gather(s["x"], cfg.K, seg, s["lay"]["row_of_slot"], s["W"][0], s["W"][1], ws)
        else:
            hub.moe_ffn_gate_up(s["xp"], seg, s["W"][0], s["W"][1], ws)
        torch.cuda.synchronize()
        got.append(ws[:a_bytes].clone())
        del ws
    assert torch.equal(got[0], got[1])
    assert bool(got[0].any())


def test_full_combine_of_identity_experts_returns_input(G, S):
    """Holds at any size: with y = xp the weighted sum gives back x (weights sum to one)."""
    s = S
    cfg = s["cfg"]
    out = G.gpu_combine(s["xp"], cfg.K, s["lay"]["slot_of_row"], s["w"])
    diff = (out.float() - s["x"].float()).abs()
    ref = s["x"].float().abs()
    assert float(diff.max()) <= 2e-2 * max(1.0, float(ref.max()) / 4)
    assert float(diff.norm() / ref.norm()) <= 4e-3


def test_expert_parallel_receive_buffer_ffn(G, S):
    """The local experts' FFN at its real shape: 65536 received rows split over 8 experts by popularity."""
    import torch
    import moe_inputs.device as mid
    s = S
    if s["name"] != "dsv3_ep":
        pytest.skip("only the expert-parallel workload has a receive buffer")
    cfg = s["cfg"]
    M = cfg.R
    recv = mid.fill_normal(torch.empty((M, cfg.H), dtype=torch.bfloat16, device="cuda:0"), cfg.seed,
                           mi.STREAM_RECV_X, 0, 1.0)
    seg = np.concatenate([[0], np.cumsum(mi.recv_segment_counts(cfg, M, 0))]).astype(np.int32)
    y = G.gpu_ffn(recv, mid.to_device(seg), *s["W"])
    rng = np.random.default_rng(7)
    rows = _sample_rows(rng, seg, 3)
    want = _oracle_rows_by_expert(G, G.host(recv), seg, s["W"], rows)
    ma, rl = G.check_close(G.host(y[torch.from_numpy(rows).to(y.device)]), want, 2e-2, 1e-2, what="recv ffn")
    _say(f"   segments {np.diff(seg).tolist()}; max-abs {ma:.3e} rel-L2 {rl:.3e}")


def test_release_device_memory():
    import torch
    _state.clear()
    torch.cuda.empty_cache()
