"""GPU parity: every step of the HIP path, through the C ABI, against the CPU oracle
on the same seeded inputs.  Integers bit-exact; floats within the stated bar.
Sizes are small enough for the oracle to compute everything, yet span several
tiles, ragged tails and the degenerate cases of each step."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import moe_inputs as mi  # noqa: E402
import oracle  # noqa: E402


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import gpu_layer
    import paper_2605_05888_amd as hub
    hub.load_library(build_if_missing=False)   # the built HIP library must be there
    return gpu_layer


def _say(*a):
    print(*a, flush=True)


# small stand-ins with the routing structure (E, K, G, skew, score mode, dtype) of the five workloads
SMALL = {
    "tiny": mi.CONFIGS["tiny"],
    "mixtral": mi.small_variant(mi.CONFIGS["mixtral"], N=1000, H=256, F=320),
    "gptoss": mi.small_variant(mi.CONFIGS["gptoss"], N=777, H=192, F=192),
    "dsv3": mi.small_variant(mi.CONFIGS["dsv3"], N=515, H=128, F=64),
    "dsv3_ep": mi.small_variant(mi.CONFIGS["dsv3_ep"], N=300, H=128, F=128),
}


def test_device_fill_equals_host_generator(G):
    import moe_inputs.device as mid
    cfg = SMALL["gptoss"]
    for s in (mi.STREAM_X, mi.STREAM_W_ROUTER, mi.STREAM_W_GATE, mi.STREAM_W_DOWN):
        assert np.array_equal(G.host(mid.device_tensor(cfg, s)), mi.host_tensor(cfg, s)), s
    big = mi.CONFIGS["dsv3"]                       # far into a large tensor (flat index > 2^32)
    d = mid.device_tensor(big, mi.STREAM_W_UP, 200, 1)
    h = mi.host_tensor(big, mi.STREAM_W_UP, 200, 1)
    assert np.array_equal(G.host(d), h)


@pytest.mark.parametrize("name", list(SMALL))
def test_route_parity(G, name):
    import moe_inputs.device as mid
    cfg = SMALL[name]
    _say("route", cfg)
    x, Wr = mi.host_tensor(cfg, mi.STREAM_X), mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    bias = mi.router_bias(cfg)
    o_idx, o_w, o_lg = oracle.route(x, Wr, bias, cfg.K, cfg.score_mode)
    dbias = None if bias is None else mid.to_device(bias)
    for want_logits in (True, False):
        idx, w, lg = G.gpu_route(mid.to_device(x), mid.to_device(Wr), dbias, cfg.K, cfg.score_mode, want_logits)
        if want_logits:
            assert np.array_equal(G.host(lg).view(np.uint32), o_lg.view(np.uint32))   # same bits
        assert np.array_equal(G.host(idx), o_idx)
        assert np.max(np.abs(G.host(w).astype(np.float64) - o_w)) <= 2e-6


@pytest.mark.parametrize("N,H,E,K,dtype", [(1, 8, 1, 1, mi.BF16), (9, 200, 5, 5, mi.BF16), (70, 72, 12, 3, mi.F32),
                                           (33, 1000, 70, 6, mi.BF16), (5, 64, 1024, 32, mi.F32)])
def test_route_ragged_shapes_and_ties(G, N, H, E, K, dtype):
    import moe_inputs.device as mid
    import dataclasses
    cfg = dataclasses.replace(mi.CONFIGS["tiny"], N=N, H=H, E=E, K=K, dtype=dtype, seed=11)
    _say("route ragged", cfg)
    x, Wr = mi.host_tensor(cfg, mi.STREAM_X), mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    Wr = np.round(Wr * 4 * np.sqrt(H)) / 4                    # coarse weights
    if E > 2:
        Wr[:, 2] = Wr[:, 0]                                   # experts 0 and 2 always tie
    bias = np.zeros(E, np.float32)
    o_idx, o_w, o_lg = oracle.route(x, Wr, bias, K, oracle.SIGMOID_TOPK)
    idx, w, lg = G.gpu_route(mid.to_device(x), mid.to_device(Wr.astype(np.float32)), mid.to_device(bias), K,
                             oracle.SIGMOID_TOPK)
    assert np.array_equal(G.host(lg).view(np.uint32), o_lg.view(np.uint32))
    assert np.array_equal(G.host(idx), o_idx)
    assert np.max(np.abs(G.host(w).astype(np.float64) - o_w)) <= 2e-6


def _random_idx(rng, N, E, K, skew):
    p = None
    if skew:
        p = 1.0 / np.arange(1, E + 1) ** skew
        p /= p.sum()
    return np.stack([rng.choice(E, size=K, replace=False, p=p) for _ in range(N)]).astype(np.int32)


LAYOUT_CASES = [(0, 8, 2, 2, 0), (1, 1, 1, 1, 0), (3, 4, 2, 4, 0), (64, 8, 1, 1, 0), (513, 8, 2, 1, 0),
                (1000, 128, 4, 1, 1.0), (4097, 256, 8, 32, 1.2), (2000, 256, 8, 256, 0), (700, 6, 6, 3, 0),
                (300, 1000, 16, 8, 0.5), (5000, 2, 1, 2, 2.0)]


@pytest.mark.parametrize("N,E,K,Gd,skew", LAYOUT_CASES)
def test_layout_parity(G, N, E, K, Gd, skew):
    import moe_inputs.device as mid
    _say("layout", N, E, K, Gd, skew)
    rng = np.random.default_rng(N + E)
    idx = _random_idx(rng, N, E, K, skew) if N else np.zeros((0, K), np.int32)
    want = oracle.layout(idx, E, Gd)
    got = G.gpu_layout(mid.to_device(idx).reshape(N, K), E, Gd)
    for k in want:
        assert np.array_equal(G.host(got[k]), want[k]), k
    again = G.gpu_layout(mid.to_device(idx).reshape(N, K), E, Gd)    # deterministic
    for k in want:
        assert np.array_equal(G.host(again[k]), want[k]), k


@pytest.mark.parametrize("N,E,K,Gd,skew", LAYOUT_CASES)
def test_arrival_order_layout_unique_parts_exact_and_slots_valid(G, N, E, K, Gd, skew):
    """Row order inside a region is not unique: counts, offsets and destinations must equal the oracle's,
    the slot maps must be inverse bijections that keep every row inside its expert's region."""
    import moe_inputs.device as mid
    from layout_checks import check_layout_is_valid
    _say("arrival layout", N, E, K, Gd, skew)
    rng = np.random.default_rng(N + E)
    idx = _random_idx(rng, N, E, K, skew) if N else np.zeros((0, K), np.int32)
    want = oracle.layout(idx, E, Gd)
    for _ in range(2):                                           # the second call finds used counters
        got = {k: G.host(v) for k, v in G.gpu_layout_arrival(mid.to_device(idx).reshape(N, K), E, Gd).items()}
        for k in ("expert_counts", "expert_offsets", "dest_counts", "dest_offsets"):
            assert np.array_equal(got[k], want[k]), k
        check_layout_is_valid(idx, E, Gd, got)


@pytest.mark.parametrize("name", list(SMALL))
def test_route_with_rows_taken_on_arrival(G, name):
    """moe_route_resolve_arrival (the row pointer drawn in the top-K kernel, as the row is produced): routing
    outputs bit for bit those of the oracle, counts / offsets / destinations exact, slot maps a valid dense packing;
    twice, the second call over used buffers."""
    import moe_inputs.device as mid
    from layout_checks import check_layout_is_valid
    cfg = SMALL[name]
    _say("route + arrival-order resolution", cfg)
    x, Wr = mi.host_tensor(cfg, mi.STREAM_X), mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    bias = mi.router_bias(cfg)
    o_idx, o_w, o_lg = oracle.route(x, Wr, bias, cfg.K, cfg.score_mode)
    want = oracle.layout(o_idx, cfg.E, cfg.G)
    dbias = None if bias is None else mid.to_device(bias)
    dx, dWr = mid.to_device(x), mid.to_device(Wr)
    for _ in range(2):
        idx, w, lg, lay = G.gpu_route_resolve_arrival(dx, dWr, dbias, cfg.K, cfg.G, cfg.score_mode)
        assert np.array_equal(G.host(lg).view(np.uint32), o_lg.view(np.uint32))
        assert np.array_equal(G.host(idx), o_idx)
        assert np.max(np.abs(G.host(w).astype(np.float64) - o_w)) <= 2e-6
        got = {k: G.host(v) for k, v in lay.items()}
        for k in ("expert_counts", "expert_offsets", "dest_counts", "dest_offsets"):
            assert np.array_equal(got[k], want[k]), k
        check_layout_is_valid(o_idx, cfg.E, cfg.G, got)


def test_route_with_rows_taken_on_arrival_no_tokens(G):
    import torch
    import paper_2605_05888_amd as hub
    E, Gd, K = 8, 2, 2
    z = lambda n, v=-7: torch.full((n,), v, dtype=torch.int32, device="cuda:0")
    cnt, off, dc, do = z(E), z(E + 1), z(Gd), z(Gd + 1)
    x = torch.zeros((0, 64), dtype=torch.bfloat16, device="cuda:0")
    Wr = torch.zeros((64, E), dtype=torch.float32, device="cuda:0")
    hub.moe_route_resolve_arrival(x, Wr, None, K, Gd, hub.SCORE_SOFTMAX_TOPK, z(0).reshape(0, K),
                                  torch.zeros((0, K), dtype=torch.float32, device="cuda:0"), cnt, off, dc, do, z(0), z(0))
    torch.cuda.synchronize()
    assert not cnt.any() and not off.any() and not dc.any() and not do.any()


def test_arrival_order_layout_all_rows_to_one_expert(G):
    import moe_inputs.device as mid
    from layout_checks import check_layout_is_valid
    idx = np.full((3000, 1), 37, np.int32)                       # one row pointer takes every arrival
    got = {k: G.host(v) for k, v in G.gpu_layout_arrival(mid.to_device(idx), 64, 8).items()}
    check_layout_is_valid(idx, 64, 8, got)


def test_layout_all_rows_to_one_expert(G):
    import moe_inputs.device as mid
    idx = np.full((3000, 1), 37, np.int32)
    want = oracle.layout(idx, 64, 8)
    got = G.gpu_layout(mid.to_device(idx), 64, 8)
    for k in want:
        assert np.array_equal(G.host(got[k]), want[k]), k


@pytest.mark.parametrize("name", list(SMALL))
def test_permute_and_combine_parity(G, name):
    import moe_inputs.device as mid
    cfg = SMALL[name]
    _say("permute/combine", cfg)
    x = mi.host_tensor(cfg, mi.STREAM_X)
    rng = np.random.default_rng(cfg.seed)
    idx = _random_idx(rng, cfg.N, cfg.E, cfg.K, cfg.zipf_s)
    lay = oracle.layout(idx, cfg.E, cfg.G)
    dlay = {k: mid.to_device(v) for k, v in lay.items()}
    xp = G.gpu_permute(mid.to_device(x), cfg.K, dlay)
    want_xp = oracle.permute(x, cfg.K, lay["slot_of_row"])
    assert np.array_equal(G.host(xp), want_xp)                       # bitwise
    w = rng.random((cfg.N, cfg.K))
    w /= w.sum(axis=1, keepdims=True)
    w32 = w.astype(np.float32)
    # combine over identity experts (y = xp) and over unrelated y
    for y in (want_xp, mi.host_tensor(mi.small_variant(cfg, N=cfg.R, H=cfg.H, F=cfg.F), mi.STREAM_X)):
        out = G.gpu_combine(mid.to_device(y), cfg.K, dlay["slot_of_row"], mid.to_device(w32))
        want = oracle.combine(y, cfg.K, lay["slot_of_row"], w32.astype(np.float64))
        tol = (2e-2, 4e-3) if cfg.dtype == mi.BF16 else (1e-5, 1e-6)
        G.check_close(G.host(out), want, *tol, what="combine")


@pytest.mark.parametrize("N,H,K,dtype", [(37, 520, 2, mi.BF16), (21, 576, 16, mi.BF16), (29, 260, 2, mi.F32),
                                         (10, 8, 8, mi.BF16), (13, 2056, 3, mi.BF16), (6, 1032, 32, mi.BF16)])
def test_row_moves_with_fewer_chunks_than_copies_in_the_last_round(G, N, H, K, dtype):
    """Row lengths whose count of 16-byte chunks leaves fewer lanes in a wavefront's last round than the
    token has copies (chunks % 64 in [1, K), or the same after the four-at-a-time rounds): the slot and
    the weight of copy k must reach the lanes still at work although lane k itself is not among them."""
    import moe_inputs.device as mid
    import dataclasses
    E = max(K, 4)
    cfg = dataclasses.replace(mi.CONFIGS["tiny"], N=N, H=H, E=E, K=K, dtype=dtype, seed=77)
    _say("row moves", cfg)
    x = mi.host_tensor(cfg, mi.STREAM_X)
    rng = np.random.default_rng(H + K)
    idx = _random_idx(rng, N, E, K, 0)
    lay = oracle.layout(idx, E, 1)
    dlay = {k: mid.to_device(v) for k, v in lay.items()}
    xp = G.gpu_permute(mid.to_device(x), K, dlay)
    want_xp = oracle.permute(x, K, lay["slot_of_row"])
    assert np.array_equal(G.host(xp), want_xp)
    w = rng.random((N, K)) + 0.1
    w /= w.sum(axis=1, keepdims=True)
    w32 = w.astype(np.float32)
    y = mi.host_tensor(dataclasses.replace(cfg, N=N * K, seed=78), mi.STREAM_X)
    out = G.gpu_combine(mid.to_device(y), K, dlay["slot_of_row"], mid.to_device(w32))
    want = oracle.combine(y, K, lay["slot_of_row"], w32.astype(np.float64))
    tol = (2e-2, 4e-3) if dtype == mi.BF16 else (1e-5, 1e-6)
    G.check_close(G.host(out), want, *tol, what="combine")


@pytest.mark.parametrize("N,H,E,K,dtype", [(45, 192, 8, 2, mi.BF16), (70, 2880 // 8, 128, 4, mi.BF16),
                                           (33, 200, 12, 3, mi.F32), (64, 72, 256, 8, mi.BF16)])
def test_route_reads_nothing_outside_its_operands(G, N, H, E, K, dtype):
    """x and W_r are views into the middle of larger buffers filled with NaN; H is not a multiple of the
    router's K tile of 128, so its last tile hangs over the end of W_r and of the last token's row.
    Whatever is fetched from beyond an operand would turn logits into NaN: they must equal the oracle's
    bit for bit."""
    import moe_inputs.device as mid
    import dataclasses
    import torch
    cfg = dataclasses.replace(mi.CONFIGS["tiny"], N=N, H=H, E=E, K=K, dtype=dtype, seed=13)
    _say("route inside poisoned memory", cfg)
    x, Wr = mi.host_tensor(cfg, mi.STREAM_X), mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    bias = (np.arange(E) % 5).astype(np.float32) / 8
    o_idx, o_w, o_lg = oracle.route(x, Wr, bias, K, oracle.SOFTMAX_TOPK)
    pad = 1 << 16                                                # elements of NaN on either side
    dt = torch.bfloat16 if dtype == mi.BF16 else torch.float32
    xbuf = torch.full((pad + N * H + pad,), float("nan"), dtype=dt, device="cuda:0")
    wbuf = torch.full((pad + H * E + pad,), float("nan"), dtype=torch.float32, device="cuda:0")
    dx = mid.to_device(x)
    xbuf[pad:pad + N * H] = (dx.view(dt) if dx.dtype != dt else dx).reshape(-1)
    wbuf[pad:pad + H * E] = mid.to_device(Wr).reshape(-1)
    xv, wv = xbuf[pad:pad + N * H].view(N, H), wbuf[pad:pad + H * E].view(H, E)
    idx, w, lg = G.gpu_route(xv, wv, mid.to_device(bias), K, oracle.SOFTMAX_TOPK)
    assert np.array_equal(G.host(lg).view(np.uint32), o_lg.view(np.uint32))
    assert np.array_equal(G.host(idx), o_idx)
    assert np.max(np.abs(G.host(w).astype(np.float64) - o_w)) <= 2e-6


def _segments(rng, M, E, empty=()):
    cuts = np.sort(rng.integers(0, M + 1, size=E - 1))
    seg = np.concatenate([[0], cuts, [M]]).astype(np.int32)
    for e in empty:
        seg[e + 1] = seg[e]
    seg = np.maximum.accumulate(seg)
    seg[-1] = M
    return seg


# the grouped GEMM has two tile geometries (experts with at most 64 rows, and the rest), draws
# tiles at run time and carries on from one tile into the next when the reduction has three K
# tiles of 64 or more: the cases mix expert sizes and put H and F on both sides of that length
FFN_CASES = [  # M, H, F, E_local, dtype, empty experts
    (300, 128, 192, 5, mi.BF16, (1,)),        # small-tile plan, ragged rows and columns
    (1500, 256, 320, 3, mi.BF16, ()),         # big-tile plan, several row tiles, F not a tile multiple
    (900, 64, 64, 1, mi.BF16, ()),            # one expert
    (130, 192, 448, 40, mi.BF16, (0, 7, 39)), # many tiny experts, some empty
    (2600, 576, 128, 6, mi.BF16, (2,)),       # long first reduction, short second; big and small experts
    (700, 64, 640, 9, mi.BF16, ()),           # short first reduction (one K tile), long second
    (3000, 128, 64, 1024, mi.BF16, tuple(range(5, 1024, 7))),  # the largest expert count the schedule takes
    (512, 128, 256, 8, mi.F32, ()),           # fp32 path
    (77, 36, 20, 3, mi.F32, (1,)),            # fp32, odd sizes
]


@pytest.mark.parametrize("M,H,F,E,dtype,empty", FFN_CASES)
def test_grouped_ffn_parity(G, M, H, F, E, dtype, empty):
    import moe_inputs.device as mid
    import dataclasses
    cfg = dataclasses.replace(mi.CONFIGS["tiny"], N=M, H=H, F=F, E=E, K=1, dtype=dtype, seed=21)
    _say("ffn", cfg)
    rng = np.random.default_rng(M)
    seg = _segments(rng, M, E, empty)
    xp = mi.host_tensor(cfg, mi.STREAM_X)
    Wg, Wu, Wd = (mi.host_tensor(cfg, s) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    want = oracle.ffn_rows(xp, seg, Wg, Wu, Wd)
    y = G.gpu_ffn(mid.to_device(xp), mid.to_device(seg), mid.to_device(Wg), mid.to_device(Wu), mid.to_device(Wd))
    ma, rl = G.check_close(G.host(y), want, *G.tolerances(cfg), what="ffn")
    _say("   max-abs %.3e rel-L2 %.3e" % (ma, rl))


@pytest.mark.parametrize("seed", range(6))
def test_grouped_ffn_random_segmentations(G, seed):
    """Expert sizes drawn around the tile boundaries (multiples of 256 plus or minus a few dozen rows, tiny
    and empty experts in between): every mix of full, ragged, tall and shallow tiles, tiles chained or not
    (H and F on both sides of three K tiles), against the oracle and, bit for bit, against a second run."""
    import moe_inputs.device as mid
    import dataclasses
    rng = np.random.default_rng(1000 + seed)
    E = int(rng.integers(3, 24))
    rows = []
    for _ in range(E):
        kind = rng.integers(0, 5)
        if kind == 0:
            rows.append(int(rng.integers(0, 70)))                                   # shallow or empty
        elif kind == 1:
            rows.append(int(rng.integers(65, 256)))                                 # one ragged tile
        else:
            rows.append(int(256 * rng.integers(1, 4) + rng.integers(-70, 71)))      # around a boundary
    rows = [max(r, 0) for r in rows]
    M = sum(rows)
    H, F = [(64, 128), (128, 64), (192, 320), (320, 192), (256, 256), (448, 128)][seed]
    cfg = dataclasses.replace(mi.CONFIGS["tiny"], N=M, H=H, F=F, E=E, K=1, dtype=mi.BF16, seed=50 + seed)
    _say("ffn, random segments", rows, H, F)
    seg = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    xp = mi.host_tensor(cfg, mi.STREAM_X)
    Wg, Wu, Wd = (mi.host_tensor(cfg, s) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    args = [mid.to_device(t) for t in (xp, seg, Wg, Wu, Wd)]
    y = G.host(G.gpu_ffn(*args))
    G.check_close(y, oracle.ffn_rows(xp, seg, Wg, Wu, Wd), *G.tolerances(cfg), what="ffn, random segments")
    assert np.array_equal(G.host(G.gpu_ffn(*args)), y)
    # The down projection picks 128-column tiles when the launch can have only few tiles (judged by an upper
    # bound from M and the number of experts) and 256-column tiles otherwise; 300 empty experts in front push
    # this launch over the bound.  Every output element is the same sum in the same order: same bits.
    pad = 300
    seg_p = np.concatenate([np.zeros(pad, np.int32), seg]).astype(np.int32)
    cfg_p = dataclasses.replace(cfg, E=E + pad)
    Wp = [np.concatenate([mi.host_tensor(cfg_p, s, 0, pad), w]) for s, w in
          ((mi.STREAM_W_GATE, Wg), (mi.STREAM_W_UP, Wu), (mi.STREAM_W_DOWN, Wd))]
    y_p = G.host(G.gpu_ffn(args[0], mid.to_device(seg_p), *[mid.to_device(w) for w in Wp]))
    assert np.array_equal(y_p, y)


def test_ffn_remainder_rows_riding_with_the_last_full_tile(G):
    """An expert's remainder of up to 64 rows is computed by its last full tile, in other registers and by
    other instructions than the tile's own 256 rows.  Sizes on both sides of every boundary; the result
    must be within tolerance of the oracle, must not depend on which rows of an expert are the remainder
    (segment reversed: same bits per row), and the gather form must give the same bits as permute + GEMM1."""
    import moe_inputs.device as mid
    import dataclasses
    import torch
    import paper_2605_05888_amd as hub
    rows = [257, 287, 288, 289, 320, 321, 513, 832, 64, 65, 256, 255, 0, 300]
    E, M = len(rows), sum(rows)
    cfg = dataclasses.replace(mi.CONFIGS["tiny"], N=M, H=320, F=384, E=E, K=1, dtype=mi.BF16, seed=33)
    _say("ffn, tall tiles", cfg)
    seg = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    xp = mi.host_tensor(cfg, mi.STREAM_X)
    Wg, Wu, Wd = (mi.host_tensor(cfg, s) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    dWg, dWu, dWd, dseg = (mid.to_device(t) for t in (Wg, Wu, Wd, seg))
    y = G.host(G.gpu_ffn(mid.to_device(xp), dseg, dWg, dWu, dWd))
    o_y = oracle.ffn_rows(xp, seg, Wg, Wu, Wd)
    G.check_close(y, o_y, *G.tolerances(cfg), what="ffn with tall tiles")
    # every segment reversed: the remainder rows are now computed as ordinary rows of a full tile
    rev = np.concatenate([np.arange(seg[e], seg[e + 1])[::-1] for e in range(E)]).astype(np.int32)
    y_rev = G.host(G.gpu_ffn(mid.to_device(np.ascontiguousarray(xp[rev])), dseg, dWg, dWu, dWd))
    assert np.array_equal(y_rev, y[rev])
    # the same through the gather form of GEMM1: x holds the rows in reversed order, row_of_slot undoes it
    code, dt = hub.BF16, torch.bfloat16
    nb = hub.workspace_bytes(hub.OP_GROUPED_FFN, N=M, H=cfg.H, E=E, F=cfg.F, dtype=code)
    ws = torch.zeros(nb, dtype=torch.uint8, device="cuda:0")
    yg = torch.zeros((M, cfg.H), dtype=dt, device="cuda:0")
    dx = mid.to_device(np.ascontiguousarray(xp[rev]))
    hub.moe_ffn_schedule(code, M, cfg.H, cfg.F, dseg, ws)
    hub.moe_ffn_gate_up_gather(dx.view(dt) if dx.dtype != dt else dx, 1, dseg, mid.to_device(rev), dWg, dWu, ws)
    hub.moe_ffn_down(dseg, dWd, yg, ws)
    torch.cuda.synchronize()
    assert np.array_equal(G.host(yg), y)
    # and through the down GEMM that adds its rows into the tokens' sums (K = 1: token r gets slot m's
    # row times its weight, r = rev[m]), whose epilogue has its own code for the remainder rows
    rng = np.random.default_rng(7)
    w = (0.5 + rng.random(M)).astype(np.float32)
    sums = torch.empty((M, cfg.H), dtype=torch.float32, device="cuda:0")
    out = torch.zeros((M, cfg.H), dtype=dt, device="cuda:0")
    hub.moe_ffn_down_combine(1, dseg, dWd, mid.to_device(rev), mid.to_device(w).reshape(M, 1), sums, out, ws)
    torch.cuda.synchronize()
    want = np.empty((M, cfg.H))
    want[rev] = w[rev, None].astype(np.float64) * o_y
    G.check_close(G.host(out), want, *G.tolerances(cfg), what="rows added into the sums")


def test_ffn_steps_rerun_after_one_schedule(G):
    """The tile counters are handed back by the GEMM itself: after one moe_ffn_schedule the two
    GEMM steps can be launched again and again, and moe_grouped_ffn gives the same bits."""
    import moe_inputs.device as mid
    import dataclasses
    import torch
    import paper_2605_05888_amd as hub
    cfg = dataclasses.replace(mi.CONFIGS["mixtral"], N=1800, H=320, F=384, E=7, K=1, seed=9)
    rng = np.random.default_rng(3)
    seg = _segments(rng, cfg.N, cfg.E, (4,))
    seg[1] = seg[0] + 20                                    # a 20-row expert next to big ones
    seg = np.maximum.accumulate(seg)
    xp = mid.to_device(mi.host_tensor(cfg, mi.STREAM_X))
    Wg, Wu, Wd = (mid.to_device(mi.host_tensor(cfg, s)) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    dseg = mid.to_device(seg)
    ref = G.host(G.gpu_ffn(xp, dseg, Wg, Wu, Wd)).tobytes()
    ws = torch.zeros(hub.workspace_bytes(hub.OP_GROUPED_FFN, N=cfg.N, H=cfg.H, E=cfg.E, F=cfg.F), dtype=torch.uint8,
                     device="cuda:0")
    hub.moe_ffn_schedule(hub.BF16, cfg.N, cfg.H, cfg.F, dseg, ws)
    for _ in range(3):
        y = torch.zeros((cfg.N, cfg.H), dtype=torch.bfloat16, device="cuda:0")
        hub.moe_ffn_gate_up(xp, dseg, Wg, Wu, ws)
        hub.moe_ffn_gate_up(xp, dseg, Wg, Wu, ws)           # twice in a row over the same table
        hub.moe_ffn_down(dseg, Wd, y, ws)
        torch.cuda.synchronize()
        assert G.host(y).tobytes() == ref


def _ffn_three_ways(G, cfg, seg, launches=3):
    """y of moe_ffn_gate_up + moe_ffn_down, and of `launches` runs of moe_ffn_gate_up_down over one schedule."""
    import moe_inputs.device as mid
    import torch
    import paper_2605_05888_amd as hub
    M, H, F, E = cfg.N, cfg.H, cfg.F, cfg.E
    xp = mid.to_device(mi.host_tensor(cfg, mi.STREAM_X))
    Wg, Wu, Wd = (mid.to_device(mi.host_tensor(cfg, s)) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    dseg = mid.to_device(seg)
    ws = torch.zeros(hub.workspace_bytes(hub.OP_GROUPED_FFN, N=M, H=H, E=E, F=F), dtype=torch.uint8, device="cuda:0")
    hub.moe_ffn_schedule(hub.BF16, M, H, F, dseg, ws)
    y0 = torch.zeros((M, H), dtype=torch.bfloat16, device="cuda:0")
    hub.moe_ffn_gate_up(xp, dseg, Wg, Wu, ws)
    hub.moe_ffn_down(dseg, Wd, y0, ws)
    ys = []
    for _ in range(launches):
        y = torch.zeros((M, H), dtype=torch.bfloat16, device="cuda:0")
        ws[:M * F * 2].zero_()                                   # the activation of the run before must not help
        hub.moe_ffn_gate_up_down(xp, dseg, Wg, Wu, Wd, y, ws)
        ys.append(y)
    hub.moe_ffn_status(hub.BF16, M, H, F, E, ws)
    return G.host(y0), [G.host(y) for y in ys]


@pytest.mark.parametrize("M,H,F,E,dtype,empty", [c for c in FFN_CASES if c[4] == mi.BF16])
def test_both_gemms_in_one_launch_give_the_bits_of_two_launches(G, M, H, F, E, dtype, empty):
    """The dependency-driven form (tiles of the down projection start as their rows arrive) against the two
    separate launches: same bits, also when launched again over the same schedule (the arrival counters
    count on from launch to launch)."""
    import dataclasses
    cfg = dataclasses.replace(mi.CONFIGS["tiny"], N=M, H=H, F=F, E=E, K=1, dtype=dtype, seed=21)
    _say("ffn in one launch", cfg)
    seg = _segments(np.random.default_rng(M), M, E, empty)
    y0, ys = _ffn_three_ways(G, cfg, seg)
    assert y0.any()
    for y in ys:
        assert np.array_equal(y, y0)


def test_one_launch_ffn_with_many_more_tiles_than_workgroups(G):
    """Several rounds of tiles per workgroup in both GEMMs (about 1500 and 700 tiles on 256 workgroups), big,
    tall, ragged and shallow tiles mixed: down-projection tiles are drawn while gate/up tiles still run."""
    import dataclasses
    rng = np.random.default_rng(99)
    rows = [int(r) for r in rng.choice([3, 40, 64, 65, 200, 256, 270, 300, 512, 530, 777], size=48)]
    M = sum(rows)
    cfg = dataclasses.replace(mi.CONFIGS["tiny"], N=M, H=512, F=896, E=len(rows), K=1, dtype=mi.BF16, seed=61)
    _say("ffn in one launch, many tiles", rows)
    seg = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    y0, ys = _ffn_three_ways(G, cfg, seg, launches=4)
    for y in ys:
        assert np.array_equal(y, y0)
    xp = mi.host_tensor(cfg, mi.STREAM_X)
    Wg, Wu, Wd = (mi.host_tensor(cfg, s) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    sample = np.unique(np.concatenate([seg[:-1][np.diff(seg) > 0], seg[1:][np.diff(seg) > 0] - 1,
                                       rng.integers(0, M, size=200)]))
    G.check_close(ys[0][sample], oracle.ffn_rows(xp, seg, Wg, Wu, Wd, rows=sample), 2e-2, 1e-2, what="one-launch ffn")


def test_one_launch_ffn_gives_up_at_its_poll_limit_and_says_so(G):
    """The bounded wait, forced from the host: one row tile, 300 gate/up column tiles on 256 workgroups, so
    the down-projection tiles are drawn while the second round of gate/up tiles has not even started, and a
    limit of one poll is reached.  The kernel must exit normally, the call returns MOE_OK, and
    moe_ffn_status reports the state; a normal launch afterwards is complete and correct."""
    import moe_inputs.device as mid
    import dataclasses
    import torch
    import paper_2605_05888_amd as hub
    M, H, F, E = 200, 512, 128 * 300, 1
    cfg = dataclasses.replace(mi.CONFIGS["tiny"], N=M, H=H, F=F, E=E, K=1, dtype=mi.BF16, seed=62)
    _say("ffn in one launch, poll limit", cfg)
    xp = mid.to_device(mi.host_tensor(cfg, mi.STREAM_X))
    Wg, Wu, Wd = (mid.to_device(mi.host_tensor(cfg, s)) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    dseg = mid.to_device(np.array([0, M], np.int32))
    ws = torch.zeros(hub.workspace_bytes(hub.OP_GROUPED_FFN, N=M, H=H, E=E, F=F), dtype=torch.uint8, device="cuda:0")
    hub.moe_ffn_schedule(hub.BF16, M, H, F, dseg, ws)
    y = torch.zeros((M, H), dtype=torch.bfloat16, device="cuda:0")
    hub.moe_ffn_gate_up_down(xp, dseg, Wg, Wu, Wd, y, ws, wait_limit=1)
    torch.cuda.synchronize()                                     # the kernel has exited
    with pytest.raises(hub.MoEHubError) as err:
        hub.moe_ffn_status(hub.BF16, M, H, F, E, ws)
    assert err.value.code == -5 and "waiting" in str(err.value)
    hub.moe_ffn_schedule(hub.BF16, M, H, F, dseg, ws)            # clears the word and the counters
    y2 = torch.zeros((M, H), dtype=torch.bfloat16, device="cuda:0")
    hub.moe_ffn_gate_up_down(xp, dseg, Wg, Wu, Wd, y2, ws)
    hub.moe_ffn_status(hub.BF16, M, H, F, E, ws)
    y3 = torch.zeros((M, H), dtype=torch.bfloat16, device="cuda:0")
    hub.moe_ffn_gate_up(xp, dseg, Wg, Wu, ws)
    hub.moe_ffn_down(dseg, Wd, y3, ws)
    torch.cuda.synchronize()
    assert torch.equal(y2, y3) and bool(y2.any())


def test_one_launch_ffn_refuses_activation_rows_that_share_cache_lines(G):
    """Rows of the activation that are not whole 128-byte lines (a workspace that is not 128-byte aligned)
    could leave a stale line in an XCD's L2: refused before any launch."""
    import moe_inputs.device as mid
    import torch
    import paper_2605_05888_amd as hub
    M, H, E = 300, 128, 2
    dseg = mid.to_device(np.array([0, 100, M], np.int32))
    for F, shift in ((192, 16), (192, 64)):
        _say("ffn in one launch, refused", (F, shift))
        buf = torch.zeros(hub.workspace_bytes(hub.OP_GROUPED_FFN, N=M, H=H, E=E, F=F) + 256, dtype=torch.uint8, device="cuda:0")
        ws = buf[shift:shift + buf.numel() - 256]
        xp = torch.zeros((M, H), dtype=torch.bfloat16, device="cuda:0")
        Wg = torch.zeros((E, F, H), dtype=torch.bfloat16, device="cuda:0")
        Wd = torch.zeros((E, H, F), dtype=torch.bfloat16, device="cuda:0")
        y = torch.ones((M, H), dtype=torch.bfloat16, device="cuda:0")
        hub.moe_ffn_schedule(hub.BF16, M, H, F, dseg, ws)
        with pytest.raises(hub.MoEHubError) as err:
            hub.moe_ffn_gate_up_down(xp, dseg, Wg, Wg, Wd, y, ws)
        assert err.value.code == -2 and "128-byte" in str(err.value)
        torch.cuda.synchronize()
        assert bool((y == 1).all())


@pytest.mark.parametrize("name", list(SMALL))
def test_gate_up_with_fused_gather_equals_permute_then_gate_up(G, name):
    """GEMM1 fetching its rows through row_of_slot from x gives the bits of permute + GEMM1; the whole
    chain built on it stays within the oracle's tolerance."""
    import moe_inputs.device as mid
    import torch
    import paper_2605_05888_amd as hub
    cfg = SMALL[name]
    _say("fused gather", cfg)
    dt = torch.bfloat16 if cfg.dtype == mi.BF16 else torch.float32
    code = hub.BF16 if cfg.dtype == mi.BF16 else hub.F32
    x, Wr = mi.host_tensor(cfg, mi.STREAM_X), mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    Wg, Wu, Wd = (mi.host_tensor(cfg, s) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    bias = mi.router_bias(cfg)
    dx, dWg, dWu, dWd = mid.to_device(x), mid.to_device(Wg), mid.to_device(Wu), mid.to_device(Wd)
    idx, w, _ = G.gpu_route(dx, mid.to_device(Wr), None if bias is None else mid.to_device(bias), cfg.K,
                            cfg.score_mode, want_logits=False)
    lay = G.gpu_layout(idx, cfg.E, cfg.G)
    seg = lay["expert_offsets"]
    R = cfg.N * cfg.K
    nb = hub.workspace_bytes(hub.OP_GROUPED_FFN, N=R, H=cfg.H, E=cfg.E, F=cfg.F, dtype=code)
    ys = []
    for fused in (False, True):
        ws = torch.zeros(nb, dtype=torch.uint8, device="cuda:0")
        y = torch.zeros((R, cfg.H), dtype=dt, device="cuda:0")
        hub.moe_ffn_schedule(code, R, cfg.H, cfg.F, seg, ws)
        if fused:
            hub.moe_ffn_gate_up_gather(dx.view(dt) if dx.dtype != dt else dx, cfg.K, seg, lay["row_of_slot"], dWg, dWu, ws)
        else:
            hub.moe_ffn_gate_up(G.gpu_permute(dx, cfg.K, lay), seg, dWg, dWu, ws)
        hub.moe_ffn_down(seg, dWd, y, ws)
        torch.cuda.synchronize()
        ys.append(G.host(y))
    assert ys[0].tobytes() == ys[1].tobytes()
    o_idx, o_w, _ = oracle.route(x, Wr, bias, cfg.K, cfg.score_mode)
    o_lay = oracle.layout(o_idx, cfg.E, cfg.G)
    o_y = oracle.ffn_rows(oracle.permute(x, cfg.K, o_lay["slot_of_row"]), o_lay["expert_offsets"], Wg, Wu, Wd)
    G.check_close(ys[1], o_y, *G.tolerances(cfg), what="y (fused gather)")


@pytest.mark.parametrize("name", list(SMALL))
def test_down_projection_with_combine_in_its_epilogue(G, name):
    """GEMM2 adding gate-weighted rows straight into the tokens' sums (no y, no moe_combine): the additions
    of an element come in no fixed order, so the comparison is by tolerance - against the oracle, and
    against the GPU's own moe_ffn_down + moe_combine within a few bf16 steps."""
    import moe_inputs.device as mid
    import torch
    import paper_2605_05888_amd as hub
    cfg = SMALL[name]
    if cfg.dtype != mi.BF16:
        pytest.skip("bf16 only")
    _say("down + combine fused", cfg)
    x, Wr = mi.host_tensor(cfg, mi.STREAM_X), mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    Wg, Wu, Wd = (mi.host_tensor(cfg, s) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    bias = mi.router_bias(cfg)
    o_idx, o_w, _ = oracle.route(x, Wr, bias, cfg.K, cfg.score_mode)
    o_lay = oracle.layout(o_idx, cfg.E, cfg.G)
    o_y = oracle.ffn_rows(oracle.permute(x, cfg.K, o_lay["slot_of_row"]), o_lay["expert_offsets"], Wg, Wu, Wd)
    o_out = oracle.combine(o_y, cfg.K, o_lay["slot_of_row"], o_w)
    dx, dWg, dWu, dWd = (mid.to_device(t) for t in (x, Wg, Wu, Wd))
    idx, w, _ = G.gpu_route(dx, mid.to_device(Wr), None if bias is None else mid.to_device(bias), cfg.K,
                            cfg.score_mode, want_logits=False)
    lay = G.gpu_layout(idx, cfg.E, cfg.G)
    seg, R = lay["expert_offsets"], cfg.N * cfg.K
    xp = G.gpu_permute(dx, cfg.K, lay)
    ws = torch.zeros(hub.workspace_bytes(hub.OP_GROUPED_FFN, N=R, H=cfg.H, E=cfg.E, F=cfg.F, dtype=hub.BF16),
                     dtype=torch.uint8, device="cuda:0")
    hub.moe_ffn_schedule(hub.BF16, R, cfg.H, cfg.F, seg, ws)
    hub.moe_ffn_gate_up(xp, seg, dWg, dWu, ws)
    y = torch.zeros((R, cfg.H), dtype=torch.bfloat16, device="cuda:0")
    hub.moe_ffn_down(seg, dWd, y, ws)
    ref = G.host(G.gpu_combine(y, cfg.K, lay["slot_of_row"], w))
    sums = torch.full((cfg.N, cfg.H), 7.0, dtype=torch.float32, device="cuda:0")       # the call clears it
    for _ in range(2):                                                               # and may be repeated
        out = torch.zeros((cfg.N, cfg.H), dtype=torch.bfloat16, device="cuda:0")
        hub.moe_ffn_down_combine(cfg.K, seg, dWd, lay["row_of_slot"], w, sums, out, ws)
        torch.cuda.synchronize()
        got = G.host(out)
        G.check_close(got, o_out, *G.tolerances(cfg), what="out (combine in the epilogue)")
        G.check_close(got, G.as_f64(ref), 2e-2, 4e-3, what="against moe_ffn_down + moe_combine")


def test_ffn_gemm_without_schedule_writes_nothing_and_says_so(G):
    """A workspace no schedule was built in holds no tile table: the GEMM steps leave their outputs alone
    (the calls cannot fail: nobody waits for the device), and moe_ffn_status reports it afterwards."""
    import moe_inputs.device as mid
    import dataclasses
    import torch
    import paper_2605_05888_amd as hub
    cfg = dataclasses.replace(mi.CONFIGS["mixtral"], N=300, H=128, F=128, E=2, K=1, seed=5)
    xp = mid.to_device(mi.host_tensor(cfg, mi.STREAM_X))
    Wg, Wu, Wd = (mid.to_device(mi.host_tensor(cfg, s)) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    seg = mid.to_device(np.array([0, 100, 300], np.int32))
    ws = torch.zeros(hub.workspace_bytes(hub.OP_GROUPED_FFN, N=cfg.N, H=cfg.H, E=cfg.E, F=cfg.F), dtype=torch.uint8,
                     device="cuda:0")
    a_bytes = cfg.N * cfg.F * 2
    status = lambda M: hub.moe_ffn_status(hub.BF16, M, cfg.H, cfg.F, cfg.E, ws)
    status(cfg.N)                                                        # nothing has run yet
    y = torch.full((cfg.N, cfg.H), 3.0, dtype=torch.bfloat16, device="cuda:0")
    hub.moe_ffn_gate_up(xp, seg, Wg, Wu, ws)
    hub.moe_ffn_down(seg, Wd, y, ws)
    torch.cuda.synchronize()
    assert not ws[:a_bytes].any() and bool((y == 3.0).all())
    with pytest.raises(hub.MoEHubError) as err:
        status(cfg.N)
    assert err.value.code == -5
    hub.moe_ffn_schedule(hub.BF16, cfg.N - 44, cfg.H, cfg.F, seg, ws)     # a schedule for another row count
    status(cfg.N - 44)                                                   # the schedule clears the word
    hub.moe_ffn_gate_up(xp, seg, Wg, Wu, ws)
    hub.moe_ffn_down(seg, Wd, y, ws)
    torch.cuda.synchronize()
    assert bool((y == 3.0).all())
    hub.moe_ffn_schedule(hub.BF16, cfg.N, cfg.H, cfg.F, seg, ws)          # the right one: all is well
    hub.moe_ffn_gate_up(xp, seg, Wg, Wu, ws)
    hub.moe_ffn_down(seg, Wd, y, ws)
    status(cfg.N)
    assert bool((y != 3.0).any())


def test_grouped_ffn_leaves_rows_outside_segments_untouched(G):
    import moe_inputs.device as mid
    import dataclasses
    import torch
    cfg = dataclasses.replace(mi.CONFIGS["mixtral"], N=400, H=128, F=128, E=2, K=1, seed=5)
    xp = mi.host_tensor(cfg, mi.STREAM_X)
    Wg, Wu, Wd = (mi.host_tensor(cfg, s) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    seg = np.array([10, 150, 390], np.int32)              # rows 0..9 and 390..399 belong to nobody
    y = G.gpu_ffn(mid.to_device(xp), mid.to_device(seg), mid.to_device(Wg), mid.to_device(Wu), mid.to_device(Wd))
    yh = G.host(y)
    assert not yh[:10].any() and not yh[390:].any()        # still the zeros the buffer started with
    want = oracle.ffn_rows(xp, seg, Wg, Wu, Wd, rows=np.arange(10, 390))
    G.check_close(yh[10:390], want, 2e-2, 1e-2, what="ffn inner rows")


@pytest.mark.parametrize("name", list(SMALL))
def test_whole_layer_parity(G, name):
    """route -> layout -> permute -> grouped FFN -> combine, each GPU step fed by the GPU's own outputs."""
    import moe_inputs.device as mid
    cfg = SMALL[name]
    _say("layer", cfg)
    x, Wr = mi.host_tensor(cfg, mi.STREAM_X), mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    Wg, Wu, Wd = (mi.host_tensor(cfg, s) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    bias = mi.router_bias(cfg)
    # oracle chain
    o_idx, o_w, _ = oracle.route(x, Wr, bias, cfg.K, cfg.score_mode)
    o_lay = oracle.layout(o_idx, cfg.E, cfg.G)
    o_xp = oracle.permute(x, cfg.K, o_lay["slot_of_row"])
    o_y = oracle.ffn_rows(o_xp, o_lay["expert_offsets"], Wg, Wu, Wd)
    o_out = oracle.combine(o_y, cfg.K, o_lay["slot_of_row"], o_w)
    # GPU chain
    dx = mid.to_device(x)
    idx, w, _ = G.gpu_route(dx, mid.to_device(Wr), None if bias is None else mid.to_device(bias), cfg.K,
                            cfg.score_mode, want_logits=False)
    lay = G.gpu_layout(idx, cfg.E, cfg.G)
    xp = G.gpu_permute(dx, cfg.K, lay)
    y = G.gpu_ffn(xp, lay["expert_offsets"], mid.to_device(Wg), mid.to_device(Wu), mid.to_device(Wd))
    out = G.gpu_combine(y, cfg.K, lay["slot_of_row"], w)
    assert np.array_equal(G.host(idx), o_idx)
    for k in o_lay:
        assert np.array_equal(G.host(lay[k]), o_lay[k]), k
    assert np.array_equal(G.host(xp), o_xp)
    tol = G.tolerances(cfg)
    G.check_close(G.host(y), o_y, *tol, what="y")
    ma, rl = G.check_close(G.host(out), o_out, *tol, what="out")
    _say("   out max-abs %.3e rel-L2 %.3e" % (ma, rl))


@pytest.mark.parametrize("name", list(SMALL))
def test_whole_layer_over_arrival_order_layout(G, name):
    """The layer's output does not depend on the order of rows inside a region: over the arrival-order
    layout it is bit for bit the output over the stable layout, and within tolerance of the oracle."""
    import moe_inputs.device as mid
    from layout_checks import check_layout_is_valid
    cfg = SMALL[name]
    _say("layer, arrival order", cfg)
    x, Wr = mi.host_tensor(cfg, mi.STREAM_X), mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    Wg, Wu, Wd = (mi.host_tensor(cfg, s) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    bias = mi.router_bias(cfg)
    o_idx, o_w, _ = oracle.route(x, Wr, bias, cfg.K, cfg.score_mode)
    o_lay = oracle.layout(o_idx, cfg.E, cfg.G)
    o_y = oracle.ffn_rows(oracle.permute(x, cfg.K, o_lay["slot_of_row"]), o_lay["expert_offsets"], Wg, Wu, Wd)
    o_out = oracle.combine(o_y, cfg.K, o_lay["slot_of_row"], o_w)
    dx, dWg, dWu, dWd = (mid.to_device(t) for t in (x, Wg, Wu, Wd))
    idx, w, _ = G.gpu_route(dx, mid.to_device(Wr), None if bias is None else mid.to_device(bias), cfg.K,
                            cfg.score_mode, want_logits=False)
    outs = []
    for layout in (G.gpu_layout, G.gpu_layout_arrival):
        lay = layout(idx, cfg.E, cfg.G)
        check_layout_is_valid(o_idx, cfg.E, cfg.G, {k: G.host(v) for k, v in lay.items()})
        xp = G.gpu_permute(dx, cfg.K, lay)
        assert np.array_equal(G.host(xp)[G.host(lay["slot_of_row"])], np.repeat(x, cfg.K, axis=0))
        y = G.gpu_ffn(xp, lay["expert_offsets"], dWg, dWu, dWd)
        outs.append(G.host(G.gpu_combine(y, cfg.K, lay["slot_of_row"], w)))
    assert np.array_equal(outs[0], outs[1])
    G.check_close(outs[1], o_out, *G.tolerances(cfg), what="out over arrival-order layout")


def test_expert_parallel_rank_share(G):
    """One destination's 8 local experts: FFN over rows [dest_offsets[g], dest_offsets[g+1]) only."""
    import moe_inputs.device as mid
    cfg = SMALL["dsv3_ep"]
    Eg = cfg.E // cfg.G
    g = 3
    x, Wr = mi.host_tensor(cfg, mi.STREAM_X), mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    o_idx, _, _ = oracle.route(x, Wr, mi.router_bias(cfg), cfg.K, cfg.score_mode)
    o_lay = oracle.layout(o_idx, cfg.E, cfg.G)
    o_xp = oracle.permute(x, cfg.K, o_lay["slot_of_row"])
    Wg, Wu, Wd = (mi.host_tensor(cfg, s, g * Eg, Eg) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    seg = o_lay["expert_offsets"][g * Eg:(g + 1) * Eg + 1]
    lo, hi = int(o_lay["dest_offsets"][g]), int(o_lay["dest_offsets"][g + 1])
    assert lo == seg[0] and hi == seg[-1]
    want = oracle.ffn_rows(o_xp, seg, Wg, Wu, Wd, rows=np.arange(lo, hi))
    dlay = G.gpu_layout(mid.to_device(o_idx), cfg.E, cfg.G)
    y = G.gpu_ffn(mid.to_device(o_xp), dlay["expert_offsets"][g * Eg:(g + 1) * Eg + 1].contiguous(),
                  mid.to_device(Wg), mid.to_device(Wu), mid.to_device(Wd))
    yh = G.host(y)
    G.check_close(yh[lo:hi], want, 2e-2, 1e-2, what="local experts")
    assert not yh[:lo].any() and not yh[hi:].any()


def test_error_returns_launch_nothing(G):
    import torch
    import paper_2605_05888_amd as hub
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda:0")
    xp = torch.full((8, 64), 3.0, dtype=torch.bfloat16, device="cuda:0")
    s = torch.zeros(8, dtype=torch.int32, device="cuda:0")
    lib = hub.load_library()
    rc = lib.moe_permute(x.data_ptr(), 7, 4, 64, 2, s.data_ptr(), s.data_ptr(), xp.data_ptr(), None)
    assert rc == -2 and "dtype" in hub.last_error()
    rc = lib.moe_permute(x.data_ptr(), hub.BF16, 4, 60, 2, s.data_ptr(), s.data_ptr(), xp.data_ptr(), None)
    assert rc == -1
    torch.cuda.synchronize()
    assert bool((xp == 3.0).all())                              # output untouched
    with pytest.raises(hub.MoEHubError):
        G.hub.moe_grouped_ffn(xp, s[:2].contiguous(), torch.zeros((1, 64, 64), dtype=torch.bfloat16, device="cuda:0"),
                              torch.zeros((1, 64, 64), dtype=torch.bfloat16, device="cuda:0"),
                              torch.zeros((1, 64, 64), dtype=torch.bfloat16, device="cuda:0"),
                              torch.zeros_like(xp), None)       # missing workspace


def test_repeated_calls_are_bit_identical(G):
    """No atomics and no order dependence anywhere on the path: two runs give the same bits."""
    import moe_inputs.device as mid
    cfg = SMALL["gptoss"]
    x, Wr = mi.host_tensor(cfg, mi.STREAM_X), mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    Wg, Wu, Wd = (mid.to_device(mi.host_tensor(cfg, s)) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    dx, dWr, db = mid.to_device(x), mid.to_device(Wr), mid.to_device(mi.router_bias(cfg))
    runs = []
    for _ in range(3):
        idx, w, lg = G.gpu_route(dx, dWr, db, cfg.K, cfg.score_mode)
        lay = G.gpu_layout(idx, cfg.E, cfg.G)
        xp = G.gpu_permute(dx, cfg.K, lay)
        y = G.gpu_ffn(xp, lay["expert_offsets"], Wg, Wu, Wd)
        out = G.gpu_combine(y, cfg.K, lay["slot_of_row"], w)
        runs.append([G.host(t).tobytes() for t in (idx, w, lg, lay["slot_of_row"], lay["row_of_slot"], xp, y, out)])
    assert runs[0] == runs[1] == runs[2]
