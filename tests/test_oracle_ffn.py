"""Pins for the oracle's expert computation (two GEMMs with a gated activation)."""
import numpy as np
import pytest

import moe_inputs as mi
import oracle


def _dense_swiglu(x, Wg, Wu, Wd):
    """Textbook form with float64 library matmuls; weights are out x in."""
    g = x @ Wg.T
    u = x @ Wu.T
    return (g / (1.0 + np.exp(-g)) * u) @ Wd.T


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def test_single_expert_is_a_dense_gated_mlp():
    rng = np.random.default_rng(0)
    M, H, F = 13, 24, 40                     # H != F: transposed operands cannot pass
    x, Wg, Wu, Wd = _rand(rng, M, H), _rand(rng, 1, F, H), _rand(rng, 1, F, H), _rand(rng, 1, H, F)
    y = oracle.ffn_rows(x, [0, M], Wg, Wu, Wd)
    assert np.allclose(y, _dense_swiglu(x, Wg[0], Wu[0], Wd[0]), rtol=1e-12, atol=1e-12)


def test_gate_and_up_are_not_interchangeable():
    rng = np.random.default_rng(1)
    M, H, F = 5, 8, 12
    x, Wg, Wu, Wd = _rand(rng, M, H), _rand(rng, 1, F, H), _rand(rng, 1, F, H), _rand(rng, 1, H, F)
    y = oracle.ffn_rows(x, [0, M], Wg, Wu, Wd)
    swapped = _dense_swiglu(x, Wu[0], Wg[0], Wd[0])
    assert np.max(np.abs(y - swapped)) > 1e-3            # silu applies to the gate branch only
    # closed form on a 1x1x1 case: silu(2*3) * (2*5) * 7
    y1 = oracle.ffn_rows(np.array([[2.0]]), [0, 1], np.array([[[3.0]]]), np.array([[[5.0]]]), np.array([[[7.0]]]))
    assert np.isclose(y1[0, 0], 6.0 / (1.0 + np.exp(-6.0)) * 10.0 * 7.0, rtol=1e-15)


def test_every_segment_uses_its_own_expert():
    rng = np.random.default_rng(2)
    H, F, E = 16, 20, 5
    seg = np.array([0, 4, 4, 9, 10, 17], np.int32)       # one empty segment
    M = int(seg[-1])
    x, Wg, Wu, Wd = _rand(rng, M, H), _rand(rng, E, F, H), _rand(rng, E, F, H), _rand(rng, E, H, F)
    y = oracle.ffn_rows(x, seg, Wg, Wu, Wd)
    for e in range(E):
        lo, hi = seg[e], seg[e + 1]
        assert np.allclose(y[lo:hi], _dense_swiglu(x[lo:hi], Wg[e], Wu[e], Wd[e]), rtol=1e-12, atol=1e-12)
    rows = np.array([16, 0, 9, 3], np.int64)
    assert np.array_equal(oracle.ffn_rows(x, seg, Wg, Wu, Wd, rows=rows), y[rows])


def test_linearity_zero_and_equivariance():
    rng = np.random.default_rng(3)
    M, H, F, E = 12, 8, 10, 2
    seg = np.array([0, 7, 12], np.int32)
    x, Wg, Wu, Wd = _rand(rng, M, H), _rand(rng, E, F, H), _rand(rng, E, F, H), _rand(rng, E, H, F)
    y = oracle.ffn_rows(x, seg, Wg, Wu, Wd)
    assert np.array_equal(oracle.ffn_rows(x, seg, Wg, np.zeros_like(Wu), Wd), np.zeros_like(y))
    assert np.allclose(oracle.ffn_rows(x, seg, Wg, Wu, -2.5 * Wd), -2.5 * y, rtol=1e-12, atol=1e-12)
    assert np.allclose(oracle.ffn_rows(x, seg, Wg, 3.0 * Wu, Wd), 3.0 * y, rtol=1e-12, atol=1e-12)
    perm = np.concatenate([rng.permutation(7), 7 + rng.permutation(5)])   # inside segments
    assert np.allclose(oracle.ffn_rows(x[perm], seg, Wg, Wu, Wd), y[perm], rtol=1e-13, atol=1e-13)


def test_bf16_and_f32_storage_are_read_exactly():
    cfg = mi.small_variant(mi.CONFIGS["mixtral"], N=8, H=32, F=48)
    x = mi.host_tensor(cfg, mi.STREAM_X)                  # uint16 bf16 bit patterns
    Wg, Wu, Wd = (mi.host_tensor(cfg, s, 0, 2) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))
    seg = np.array([0, 3, 8], np.int32)
    y = oracle.ffn_rows(x, seg, Wg, Wu, Wd)
    f = lambda b: mi.bf16_bits_to_f32(b).astype(np.float64)
    y64 = oracle.ffn_rows(f(x), seg, f(Wg), f(Wu), f(Wd))
    assert np.array_equal(y, y64)
    y32 = oracle.ffn_rows(mi.bf16_bits_to_f32(x), seg, *(mi.bf16_bits_to_f32(w) for w in (Wg, Wu, Wd)))
    assert np.array_equal(y, y32)


def test_whole_layer_single_expert_top1_is_the_plain_ffn():
    # E = 1, K = 1: routing, layout, permute and combine are all identities.
    rng = np.random.default_rng(5)
    N, H, F = 10, 16, 12
    x = rng.standard_normal((N, H)).astype(np.float32)
    Wr = rng.standard_normal((H, 1)).astype(np.float32)
    idx, w, _ = oracle.route(x, Wr, None, 1, oracle.SIGMOID_TOPK)
    lay = oracle.layout(idx, 1, 1)
    xp = oracle.permute(x, 1, lay["slot_of_row"])
    Wg, Wu, Wd = _rand(rng, 1, F, H), _rand(rng, 1, F, H), _rand(rng, 1, H, F)
    y = oracle.ffn_rows(xp.astype(np.float64), lay["expert_offsets"], Wg, Wu, Wd)
    out = oracle.combine(y, 1, lay["slot_of_row"], w)
    assert np.allclose(out, _dense_swiglu(x.astype(np.float64), Wg[0], Wu[0], Wd[0]), rtol=1e-12, atol=1e-12)


def test_layer_is_invariant_to_relabelling_experts():
    cfg = mi.small_variant(mi.CONFIGS["tiny"], N=48, H=32, F=24)
    x = mi.host_tensor(cfg, mi.STREAM_X)
    Wr = mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    Wg, Wu, Wd = (mi.host_tensor(cfg, s) for s in (mi.STREAM_W_GATE, mi.STREAM_W_UP, mi.STREAM_W_DOWN))

    def layer(Wr, Wg, Wu, Wd):
        idx, w, _ = oracle.route(x, Wr, None, cfg.K, cfg.score_mode)
        lay = oracle.layout(idx, cfg.E, 1)
        xp = oracle.permute(x, cfg.K, lay["slot_of_row"])
        y = oracle.ffn_rows(xp, lay["expert_offsets"], Wg, Wu, Wd)
        return oracle.combine(y, cfg.K, lay["slot_of_row"], w)

    base = layer(Wr, Wg, Wu, Wd)
    perm = np.random.default_rng(6).permutation(cfg.E)
    moved = layer(np.ascontiguousarray(Wr[:, perm]), Wg[perm], Wu[perm], Wd[perm])
    assert np.allclose(base, moved, rtol=1e-12, atol=1e-12)
    assert np.max(np.abs(base)) > 1e-2
