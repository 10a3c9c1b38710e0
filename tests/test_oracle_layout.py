"""Pins for the oracle's mediation step (counts, offsets, slots) and row moves."""
import os

import numpy as np
import pytest

import moe_inputs as mi
import oracle
from layout_checks import check_layout_is_valid


def _read_golden(path):
    vals = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            k, *v = line.split()
            vals.setdefault(k, []).extend(int(t) for t in v)
    return vals


def test_hand_worked_two_gpu_example(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "two_gpu_four_expert_top2.txt"))
    N, K, E, G = g["N"][0], g["K"][0], g["E"][0], g["G"][0]
    idx = np.array(g["topk_idx"], np.int32).reshape(N, K)
    lay = oracle.layout(idx, E, G)
    for name in ("expert_counts", "expert_offsets", "dest_counts", "dest_offsets",
                 "row_of_slot", "slot_of_row"):
        assert list(lay[name]) == g[name], name


def _random_idx(rng, N, E, K, skew=False):
    """K distinct experts per token."""
    p = None
    if skew:
        p = 1.0 / np.arange(1, E + 1)
        p /= p.sum()
    return np.stack([rng.choice(E, size=K, replace=False, p=p) for _ in range(N)]).astype(np.int32)


@pytest.mark.parametrize("N,E,K,G,skew", [(1, 4, 2, 2, False), (37, 8, 2, 1, False), (200, 16, 4, 16, True),
                                          (333, 64, 8, 8, True), (64, 6, 6, 3, False), (50, 128, 4, 2, True)])
def test_layout_against_library_routines_and_bruteforce(N, E, K, G, skew):
    rng = np.random.default_rng(N * 7 + E)
    idx = _random_idx(rng, N, E, K, skew)
    lay = oracle.layout(idx, E, G)
    flat = idx.ravel()
    R = N * K
    cnt = np.bincount(flat, minlength=E)
    assert np.array_equal(lay["expert_counts"], cnt)
    assert lay["expert_counts"].sum() == R                       # nothing dropped
    assert np.array_equal(lay["expert_offsets"], np.concatenate([[0], np.cumsum(cnt)]))
    assert np.array_equal(lay["row_of_slot"], np.argsort(flat, kind="stable"))
    # bijection onto the R slots, mutual inverses
    assert np.array_equal(np.sort(lay["slot_of_row"]), np.arange(R))
    assert np.array_equal(lay["row_of_slot"][lay["slot_of_row"]], np.arange(R))
    # O(R^2) rank count straight from the definition of the order (expert, then flat row)
    for r in range(R):
        e = flat[r]
        want = np.count_nonzero(flat < e) + np.count_nonzero(flat[:r] == e)
        assert lay["slot_of_row"][r] == want
    # destinations: blocks of E/G consecutive experts
    Eg = E // G
    assert np.array_equal(lay["dest_counts"], cnt.reshape(G, Eg).sum(axis=1))
    assert np.array_equal(lay["dest_offsets"][:-1], lay["expert_offsets"][0:E:Eg])
    assert lay["dest_offsets"][-1] == R
    # stability: inside each expert region source rows increase
    for e in range(E):
        seg = lay["row_of_slot"][lay["expert_offsets"][e]:lay["expert_offsets"][e + 1]]
        assert np.all(np.diff(seg) > 0)
        assert np.all(flat[seg] == e)


def test_layout_degenerate_cases():
    lay = oracle.layout(np.zeros((0, 2), np.int32), 4, 2)        # no tokens
    assert list(lay["expert_offsets"]) == [0] * 5 and lay["slot_of_row"].size == 0
    idx = np.full((10, 1), 3, np.int32)                          # everything to one expert
    lay = oracle.layout(idx, 4, 4)
    assert list(lay["expert_counts"]) == [0, 0, 0, 10]
    assert list(lay["dest_offsets"]) == [0, 0, 0, 0, 10]
    assert np.array_equal(lay["slot_of_row"], np.arange(10))
    idx = np.tile(np.arange(5, dtype=np.int32), (3, 1))          # K = E: every expert, every token
    lay = oracle.layout(idx, 5, 1)
    assert list(lay["expert_counts"]) == [3] * 5
    assert np.array_equal(lay["row_of_slot"].reshape(5, 3), np.arange(15).reshape(3, 5).T)


@pytest.mark.parametrize("N,E,K,G,skew", [(1, 4, 2, 2, False), (41, 8, 2, 4, False), (300, 32, 4, 8, True),
                                          (120, 128, 8, 1, True)])
def test_arrival_order_layout_is_the_stable_sort_of_the_arrival_sequence(N, E, K, G, skew):
    """Row pointers that count arrivals (Section IV-A3) pack each region in arrival order: listing the
    rows in arrival order and sorting them stably by expert (a library routine) gives row_of_slot."""
    rng = np.random.default_rng(N + 31 * E)
    idx = _random_idx(rng, N, E, K, skew)
    flat = idx.ravel()
    R = N * K
    stable = oracle.layout(idx, E, G)
    for order in ("identity", "reversed", "random"):
        arrival = {"identity": np.arange(R), "reversed": np.arange(R)[::-1],
                   "random": rng.permutation(R)}[order].astype(np.int32)
        lay = oracle.layout_arrival(idx, E, G, arrival)
        check_layout_is_valid(idx, E, G, lay)
        assert np.array_equal(lay["row_of_slot"], arrival[np.argsort(flat[arrival], kind="stable")]), order
        for name in ("expert_counts", "expert_offsets", "dest_counts", "dest_offsets"):
            assert np.array_equal(lay[name], stable[name]), (order, name)     # order never moves a region
        if order == "identity":                                               # in-order arrival = the stable layout
            assert np.array_equal(lay["slot_of_row"], stable["slot_of_row"])
        if order == "reversed":                                               # regions hold descending rows
            for e in range(E):
                seg = lay["row_of_slot"][lay["expert_offsets"][e]:lay["expert_offsets"][e + 1]]
                assert np.all(np.diff(seg) < 0)
    # the local row id of a row is the number of earlier arrivals at its expert (brute force)
    pos = np.empty(R, np.int64)
    pos[arrival] = np.arange(R)
    for r in range(min(R, 200)):
        earlier = np.count_nonzero((flat == flat[r]) & (pos < pos[r]))
        assert lay["slot_of_row"][r] == lay["expert_offsets"][flat[r]] + earlier


def test_validity_check_rejects_planted_mistakes():
    rng = np.random.default_rng(5)
    N, E, K, G = 50, 8, 2, 2
    idx = _random_idx(rng, N, E, K)
    good = oracle.layout_arrival(idx, E, G, rng.permutation(N * K).astype(np.int32))
    check_layout_is_valid(idx, E, G, good)

    def broken(**changes):
        lay = {k: v.copy() for k, v in good.items()}
        for k, f in changes.items():
            f(lay[k])
        with pytest.raises(AssertionError):
            check_layout_is_valid(idx, E, G, lay)

    def swap_across_regions(slot):                      # two rows of different experts trade slots
        flat = idx.ravel()
        a = 0
        b = int(np.flatnonzero(flat != flat[0])[0])
        slot[a], slot[b] = slot[b], slot[a]

    def duplicate(slot):
        slot[1] = slot[0]

    def stale_inverse(row):
        row[[0, 1]] = row[[1, 0]]

    def miscount(c):
        c[0] += 1

    broken(slot_of_row=swap_across_regions)
    broken(slot_of_row=duplicate)
    broken(row_of_slot=stale_inverse)
    broken(expert_counts=miscount)
    broken(dest_offsets=miscount)
    broken(expert_offsets=lambda o: o.__setitem__(slice(1, None), o[1:] + 1))


@pytest.mark.parametrize("dtype", [np.float32, np.uint16])
def test_permute_is_a_bitwise_gather_written_once(dtype):
    rng = np.random.default_rng(3)
    N, H, E, K = 41, 24, 8, 3
    x = rng.integers(0, 60000, size=(N, H)).astype(dtype)
    idx = _random_idx(rng, N, E, K)
    lay = oracle.layout(idx, E, 1)
    xp = oracle.permute(x, K, lay["slot_of_row"])
    assert xp.shape == (N * K, H)                                # N*K*H elements in total
    assert np.array_equal(xp, x[lay["row_of_slot"] // K])        # library gather
    for r in range(N * K):
        assert xp[lay["slot_of_row"][r]].tobytes() == x[r // K].tobytes()
    # byte address of slot s is base + s * RowSize: slots never straddle rows
    assert xp.strides[0] == H * x.itemsize


def test_combine_with_identity_experts_returns_gate_weighted_input():
    cfg = mi.small_variant(mi.CONFIGS["gptoss"], N=96, H=64, F=32)
    x = mi.host_tensor(cfg, mi.STREAM_X)
    W = mi.host_tensor(cfg, mi.STREAM_W_ROUTER)
    idx, w, _ = oracle.route(x, W, mi.router_bias(cfg), cfg.K, cfg.score_mode)
    lay = oracle.layout(idx, cfg.E, cfg.G)
    xp = oracle.permute(x, cfg.K, lay["slot_of_row"])
    out = oracle.combine(xp, cfg.K, lay["slot_of_row"], w)       # experts = identity: y = xp
    xf = mi.bf16_bits_to_f32(x).astype(np.float64)
    assert np.allclose(out, xf * w.sum(axis=1, keepdims=True), rtol=1e-13, atol=1e-13)
    assert np.allclose(out, xf, rtol=1e-12, atol=1e-12)          # weights sum to one


def test_combine_matches_explicit_weighted_sum_and_pairs_weights_with_slots():
    rng = np.random.default_rng(4)
    N, H, E, K = 30, 16, 8, 3
    idx = _random_idx(rng, N, E, K)
    lay = oracle.layout(idx, E, 2)
    y = rng.standard_normal((N * K, H))
    w = rng.random((N, K))
    out = oracle.combine(y, K, lay["slot_of_row"], w)
    want = np.einsum("nk,nkh->nh", w, y[lay["slot_of_row"].reshape(N, K)])
    assert np.allclose(out, want, rtol=1e-13, atol=1e-13)
    tok = np.array([5, 0, 29], np.int64)
    assert np.array_equal(oracle.combine(y, K, lay["slot_of_row"], w, tokens=tok), out[tok])
    # y rows that are one-hot in the expert index: out[n, e] must be the weight of e for token n
    y1 = np.zeros((N * K, E))
    y1[np.arange(N * K), idx.ravel()[lay["row_of_slot"]]] = 1.0
    out1 = oracle.combine(y1, K, lay["slot_of_row"], w)
    want1 = np.zeros((N, E))
    np.put_along_axis(want1, idx.astype(np.int64), w, axis=1)
    assert np.allclose(out1, want1, atol=1e-15)
