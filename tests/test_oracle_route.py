"""Pins for the oracle's routing step (gating logits, top-K, weights).

Nothing here calls the HIP path.  Each pin compares the oracle with something
fixed outside it: exact rational arithmetic, fp64 library routines, closed
forms and crafted special cases.
"""
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import moe_inputs as mi
import oracle
from exact_f32 import add_f32, fma_f32


def _r64_exact(x_row, w_col):
    """R64 order, every operation rounded from its exact rational value."""
    p = [np.float32(0.0)] * 64
    for h in range(len(x_row)):
        p[h % 64] = fma_f32(x_row[h], w_col[h], p[h % 64])
    s = 32
    while s >= 1:
        p = [add_f32(p[l], p[l ^ s]) for l in range(64)]
        s //= 2
    return p[0]


@pytest.mark.parametrize("H", [1, 7, 64, 65, 130, 200])
def test_r64_matches_exact_rational_bruteforce(H):
    rng = np.random.default_rng(H)
    x = rng.standard_normal(H).astype(np.float32)
    w = (rng.standard_normal(H) / np.sqrt(H)).astype(np.float32)
    got = oracle.logit_r64(x, w)
    want = _r64_exact(x, w)
    assert got.tobytes() == want.tobytes()


def test_r64_bf16_input_is_widened_exactly():
    rng = np.random.default_rng(5)
    xb = mi.f32_to_bf16_bits(rng.standard_normal(192).astype(np.float32))
    w = rng.standard_normal(192).astype(np.float32)
    got = oracle.logit_r64(xb, w)
    want = _r64_exact(mi.bf16_bits_to_f32(xb), w)
    assert got.tobytes() == want.tobytes()


def test_fused_multiply_add_is_fused():
    # a*b is not representable in fp32; a fused step keeps the low bits, a
    # separate multiply then add loses them.
    a = np.float32(1.0 + 2.0 ** -12)
    b = np.float32(1.0 + 2.0 ** -12)
    c = np.float32(-(1.0 + 2.0 ** -11))
    x = np.array([a], np.float32)
    w = np.array([b], np.float32)
    # logit = fma(a, b, 0) rounds; use two terms landing in the same partial sum
    x2 = np.zeros(65, np.float32)
    w2 = np.zeros(65, np.float32)
    x2[0], w2[0] = c, 1.0          # p[0] = c
    x2[64], w2[64] = a, b          # p[0] = fma(a, b, c) = 2^-24 exactly
    got = oracle.logit_r64(x2, w2)
    assert got == np.float32(2.0 ** -24)
    assert oracle.logit_r64(x, w) == np.float32(float(a) * float(b))  # rounded product


@pytest.mark.parametrize("H,E,bf16", [(70, 3, False), (130, 5, True), (64, 2, False)])
def test_logits_with_bias_match_exact_rational_bruteforce(H, E, bf16):
    """The bias enters after the six folding rounds, as ONE fp32 addition to the folded sum: every
    operation of the whole logit, the bias add included, rounded from its exact rational value.  Biases
    are large against the last place of the sum, so a bias folded into a partial sum before the rounds
    (or added in higher precision) gives other bits."""
    rng = np.random.default_rng(100 + H)
    N = 4
    x = rng.standard_normal((N, H)).astype(np.float32)
    if bf16:
        xb = mi.f32_to_bf16_bits(x)
        x_val, x_arg = mi.bf16_bits_to_f32(xb), xb
    else:
        x_val, x_arg = x, x
    W = (rng.standard_normal((H, E)) / np.sqrt(H)).astype(np.float32)
    b = (rng.standard_normal(E) * 3).astype(np.float32)
    got = oracle.logits(x_arg, W, b)
    differs_if_folded_early = 0
    for n in range(N):
        for e in range(E):
            want = add_f32(_r64_exact(x_val[n], W[:, e]), b[e])
            assert got[n, e].tobytes() == want.tobytes(), (n, e)
            # the planted alternative: bias as the starting value of partial 0
            p = [np.float32(0.0)] * 64
            p[0] = b[e]
            for h in range(H):
                p[h % 64] = fma_f32(x_val[n, h], W[h, e], p[h % 64])
            s = 32
            while s >= 1:
                p = [add_f32(p[l], p[l ^ s]) for l in range(64)]
                s //= 2
            differs_if_folded_early += int(p[0].tobytes() != want.tobytes())
    assert differs_if_folded_early > 0          # the pin can tell the two apart on these inputs


def test_logits_close_to_fp64_dot_and_not_transposed():
    rng = np.random.default_rng(0)
    N, H, E = 9, 320, 5                     # H != E: a transposed W_r cannot pass
    x = rng.standard_normal((N, H)).astype(np.float32)
    W = (rng.standard_normal((H, E)) / np.sqrt(H)).astype(np.float32)
    b = rng.standard_normal(E).astype(np.float32)
    got = oracle.logits(x, W, b)
    want = x.astype(np.float64) @ W.astype(np.float64) + b.astype(np.float64)
    scale = np.abs(x).astype(np.float64) @ np.abs(W).astype(np.float64) + np.abs(b)
    assert np.all(np.abs(got - want) <= 1e-5 * scale)
    got_nb = oracle.logits(x, W, None)
    assert np.all(np.abs(got_nb - (want - b)) <= 1e-5 * scale)


def test_logits_one_hot_and_integer_closed_forms():
    H, E = 128, 6
    rng = np.random.default_rng(1)
    W = rng.standard_normal((H, E)).astype(np.float32)
    x = np.zeros((H, H), np.float32)
    x[np.arange(H), np.arange(H)] = 1.0      # token n is the n-th unit vector
    assert np.array_equal(oracle.logits(x, W, None), W)   # picks row n of W_r exactly
    xi = rng.integers(-8, 9, size=(4, H)).astype(np.float32)
    Wi = rng.integers(-8, 9, size=(H, E)).astype(np.float32)
    want = (xi.astype(np.int64) @ Wi.astype(np.int64)).astype(np.float32)
    assert np.array_equal(oracle.logits(xi, Wi, None), want)  # small integers: exact in any order


def _bruteforce_topk(row, K):
    order = sorted(range(len(row)), key=lambda e: (-float(row[e]), e))
    return order[:K]


@pytest.mark.parametrize("E,K", [(8, 2), (16, 4), (5, 5), (7, 1), (64, 8)])
def test_topk_equals_sorted_pairs(E, K):
    rng = np.random.default_rng(E * 100 + K)
    lg = rng.standard_normal((50, E)).astype(np.float32)
    lg[3] = np.round(lg[3])                  # many exact ties
    lg[4, :] = 0.25                          # all equal
    idx, _ = oracle.topk(lg, K, oracle.SOFTMAX_TOPK)
    for n in range(lg.shape[0]):
        assert list(idx[n]) == _bruteforce_topk(lg[n], K)


def test_topk_tie_rules():
    lg = np.full((1, 8), 1.5, np.float32)
    idx, w = oracle.topk(lg, 3, oracle.SOFTMAX_TOPK)
    assert list(idx[0]) == [0, 1, 2]                       # all equal: lowest indices
    assert np.allclose(w[0], 1.0 / 3.0, atol=1e-15)
    lg = np.array([[0.0, -0.0, 1.0, -0.0]], np.float32)    # +0 == -0: index decides
    idx, _ = oracle.topk(lg, 3, oracle.SOFTMAX_TOPK)
    assert list(idx[0]) == [2, 0, 1]
    lg = np.array([[1.0, 3.0, 3.0, 2.0]], np.float32)
    idx, _ = oracle.topk(lg, 2, oracle.SIGMOID_TOPK)
    assert list(idx[0]) == [1, 2]


def test_topk_invariants():
    rng = np.random.default_rng(7)
    N, E, K = 300, 32, 6
    lg = rng.standard_normal((N, E)).astype(np.float32)
    idx, w = oracle.topk(lg, K, oracle.SIGMOID_TOPK)
    sel = np.take_along_axis(lg, idx, axis=1)
    assert np.all(np.diff(sel, axis=1) <= 0)                   # descending preference
    for n in range(N):
        assert len(set(idx[n])) == K                           # K distinct experts
        rest = np.setdiff1d(np.arange(E), idx[n])
        assert np.all(lg[n, rest] <= sel[n, -1])               # nothing better left out
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-12)
    assert np.all(w > 0) and np.all(w <= 1)
    assert np.all(np.diff(w, axis=1) <= 1e-15)                 # monotone in the logit


def test_softmax_weights_equal_library_softmax_renormalised():
    rng = np.random.default_rng(8)
    lg = (3.0 * rng.standard_normal((40, 16))).astype(np.float32)
    K = 4
    idx, w = oracle.topk(lg, K, oracle.SOFTMAX_TOPK)
    full = scipy.special.softmax(lg.astype(np.float64), axis=1)
    sel = np.take_along_axis(full, idx, axis=1)
    assert np.allclose(w, sel / sel.sum(axis=1, keepdims=True), rtol=1e-12, atol=0)


def test_sigmoid_weights_equal_library_expit_renormalised():
    rng = np.random.default_rng(9)
    lg = (2.0 * rng.standard_normal((40, 16))).astype(np.float32)
    K = 5
    idx, w = oracle.topk(lg, K, oracle.SIGMOID_TOPK)
    s = scipy.special.expit(np.take_along_axis(lg, idx, axis=1).astype(np.float64))
    assert np.allclose(w, s / s.sum(axis=1, keepdims=True), rtol=1e-12, atol=0)
    # the two modes differ: a mode mix-up cannot pass both pins
    _, w2 = oracle.topk(lg, K, oracle.SOFTMAX_TOPK)
    assert np.max(np.abs(w - w2)) > 1e-2


def test_k_equals_one_gives_unit_weight():
    lg = np.random.default_rng(10).standard_normal((20, 8)).astype(np.float32)
    for mode in (oracle.SOFTMAX_TOPK, oracle.SIGMOID_TOPK):
        idx, w = oracle.topk(lg, 1, mode)
        assert np.array_equal(idx[:, 0], np.argmax(lg, axis=1))
        assert np.array_equal(w, np.ones((20, 1)))


def test_bias_skews_popularity_towards_zipf_head():
    cfg = mi.small_variant(mi.CONFIGS["gptoss"], N=2048, H=128, F=64)
    x = mi.host_tensor(cfg, mi.STREAM_X)
    W = mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    idx, _, _ = oracle.route(x, W, mi.router_bias(cfg), cfg.K, cfg.score_mode)
    cnt = np.bincount(idx.ravel(), minlength=cfg.E)
    p = mi.popularity(cfg)
    order = np.argsort(-p)
    assert cnt[order[:8]].sum() > 4 * cnt[order[-8:]].sum()    # head much hotter than tail
    assert cnt.sum() == cfg.N * cfg.K
