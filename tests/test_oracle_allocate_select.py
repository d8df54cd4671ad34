"""Pins for the oracle's budget apportionment, top-k selection and gather.

The apportionment rule is this build's reading of one sentence of the paper, so
it is pinned by what any such rule must satisfy plus a brute-force optimality
check of the rounding step on tiny inputs; selection and gather are pinned by
brute force and by their defining properties.
"""
import itertools
import math

import numpy as np
import pytest

from oracle import flashcache_ref as ref


# ------------------------------------------------------------------ allocation
def _check_invariants(R, T, bmin, bmax, b):
    assert int(b.sum()) == T
    assert b.min() >= bmin and b.max() <= bmax
    for i in range(len(R)):
        for j in range(len(R)):
            if R[i] > R[j]:
                assert b[i] >= b[j], (R, b)


def test_budgets_sum_bounds_monotone_random():
    rng = np.random.default_rng(0)
    for _ in range(400):
        L = int(rng.integers(1, 12))
        N = int(rng.integers(4, 300))
        bmin = int(rng.integers(1, 4))
        bmax = int(rng.integers(bmin, N + 1))
        T = int(rng.integers(L * bmin, L * bmax + 1))
        R = rng.uniform(0.0, 2.0, L) ** int(rng.integers(1, 5))
        if rng.uniform() < 0.2:
            R[rng.integers(0, L)] = 0.0
        b, margin = ref.allocate(R, T, bmin, bmax)
        _check_invariants(R, T, bmin, bmax, b)
        assert margin >= 0.0
        det = ref.allocate_detail(R, T, bmin, bmax)
        assert np.array_equal(det["budgets"], b) and det["margin"] == margin


def test_equal_ratios_split_evenly_extras_to_lowest_layers():
    b, _ = ref.allocate([0.3] * 5, 23, 1, 100)
    assert b.tolist() == [5, 5, 5, 4, 4]
    b, _ = ref.allocate([1.0] * 4, 40, 1, 100)
    assert b.tolist() == [10, 10, 10, 10]


def test_single_layer_gets_everything():
    b, _ = ref.allocate([0.123], 102, 1, 512)
    assert b.tolist() == [102]


def test_scale_invariance_and_degenerate_ratios():
    R = np.array([0.11, 0.52, 0.07, 0.9])
    a, _ = ref.allocate(R, 777, 1, 4096)
    b, _ = ref.allocate(64.0 * R, 777, 1, 4096)          # power-of-two scale: exact in fp64
    assert a.tolist() == b.tolist()
    z, _ = ref.allocate([0.0, 0.0, 0.0], 10, 1, 100)     # all-zero ratios -> uniform
    assert z.tolist() == [4, 3, 3]
    nan, _ = ref.allocate([float("nan"), 1.0], 10, 1, 100)
    assert nan.tolist() == [5, 5]


def test_clamps_redistribute():
    # layer 1 would get 90 of 100 but is capped at 50; the rest is re-shared 1:1
    b, _ = ref.allocate([1.0, 18.0, 1.0], 100, 1, 50)
    assert b.tolist() == [25, 50, 25]
    # layer 0 would get ~0 but the floor is 5; the others share the remaining 95 as 1:3
    b, _ = ref.allocate([1e-9, 1.0, 3.0], 100, 5, 100)
    assert b[0] == 5 and int(b.sum()) == 100 and b[2] > b[1]
    assert b.tolist() == [5, 24, 71]
    with pytest.raises(ValueError):
        ref.allocate([1.0, 1.0], 1, 1, 10)               # T < L*b_min
    with pytest.raises(ValueError):
        ref.allocate([1.0, 1.0], 21, 1, 10)              # T > L*b_max


def test_rounding_step_is_closest_integer_vector_brute_force():
    # without clamps the rule is largest-remainder rounding of q_l = T R_l / sum R, which
    # is the integer vector with sum T closest to q in L1 (and max-norm); check by enumeration
    rng = np.random.default_rng(5)
    for _ in range(60):
        L = int(rng.integers(2, 5))
        T = int(rng.integers(L, 13))
        R = rng.uniform(0.2, 1.0, L)
        q = T * R / R.sum()
        if q.min() < 1.0:
            continue
        b, _ = ref.allocate(R, T, 1, T)
        best = min(
            (sum(abs(c[i] - q[i]) for i in range(L)), c)
            for c in itertools.product(range(0, T + 1), repeat=L) if sum(c) == T
        )
        assert math.isclose(sum(abs(b[i] - q[i]) for i in range(L)), best[0], rel_tol=0, abs_tol=1e-9)
        assert np.all(np.abs(b - q) < 1.0)


def _random_allocation_case(rng):
    kind = int(rng.integers(0, 3))
    if kind == 0:                                  # the 28-layer workloads: similar shares, wide bounds
        L, N = 28, int(rng.choice([8192, 16384, 32768]))
        T = ref.total_budget(L, N, float(rng.choice([0.1, 0.2])))
        return rng.uniform(0.05, 0.4, L), T, 1, N
    L = int(rng.integers(2, 12))
    N = int(rng.integers(8, 400))
    bmin = int(rng.integers(1, 4))
    bmax = int(rng.integers(bmin + 1, N + 1))
    T = int(rng.integers(L * bmin, L * bmax + 1))
    R = rng.uniform(0.01, 2.0, L) ** int(rng.integers(1, 4))
    return R, T, bmin, bmax                        # kind 1 and 2 alike: clamps often bind here


def _push_pair(det, q_like, eps):
    """The perturbation that moves the shares of cliff_pair = (x, y) towards each other fastest:
    y up, x down, every other layer against the larger of the two shares."""
    x, y = det["cliff_pair"]
    e = np.full(len(q_like), -eps if q_like[y] >= q_like[x] else eps)
    e[x], e[y] = -eps, eps
    return e


def test_margin_lower_side_perturbations_below_it_never_change_budgets():
    rng = np.random.default_rng(11)
    checked = 0
    for _ in range(400):
        R, T, bmin, bmax = _random_allocation_case(rng)
        det = ref.allocate_detail(R, T, bmin, bmax)
        m = det["margin"]
        assert m >= 0.0 and det["pair_margin"] >= m
        if not (1e-12 < m < 0.5):
            continue
        tries = [rng.uniform(-1.0, 1.0, len(R)) for _ in range(4)]
        tries += [rng.choice([-1.0, 1.0], len(R)) for _ in range(6)]
        if det["cliff_pair"] is not None:
            tries += [_push_pair(det, R, 1.0), -_push_pair(det, R, 1.0)]
        for l in range(len(R)):                    # one layer against all the others
            e = -np.ones(len(R))
            e[l] = 1.0
            tries += [e, -e]
        for e in tries:
            b, _ = ref.allocate(R * (1.0 + 0.98 * m * e), T, bmin, bmax)
            assert np.array_equal(b, det["budgets"]), (R, T, bmin, bmax, m, e)
        checked += 1
    assert checked > 250


def test_margin_upper_side_hand_example_flips_the_reported_pair():
    # shares 10 * (1, 1.04, 2) / 4.04 = 2.4752, 2.5743, 4.9505: floors 2, 2, 4 and two left-over rows,
    # which go to layer 2 (.95) and layer 1 (.574); layer 0 (.475) is the first to be left out
    det = ref.allocate_detail([1.0, 1.04, 2.0], 10, 1, 10)
    assert det["budgets"].tolist() == [2, 3, 5]
    assert det["cliff_pair"] == (1, 0) and det["cliff_kind"] == "pair"
    g, q1 = 10.0 * 0.04 / 4.04, 10.4 / 4.04
    assert math.isclose(det["margin"], g / (2.0 * q1 + g), rel_tol=1e-12)
    assert math.isclose(det["margin"], 0.018868, rel_tol=1e-4)
    # layer 0 up, layer 1 down, layer 2 with layer 0 (share 1 is the larger of the pair): nothing
    # happens below the margin, and a few percent above it exactly one row moves from 1 to 0
    R = np.array([1.0, 1.04, 2.0])
    e = np.array([1.0, -1.0, 1.0])
    below, _ = ref.allocate(R * (1.0 + 0.99 * det["margin"] * e), 10, 1, 10)
    above, _ = ref.allocate(R * (1.0 + 1.05 * det["margin"] * e), 10, 1, 10)
    assert below.tolist() == [2, 3, 5]
    assert above.tolist() == [3, 2, 5]


def test_margin_upper_side_random_cases_flip_exactly_the_reported_pair():
    rng = np.random.default_rng(12)
    flipped = 0
    for _ in range(300):
        L, N = 28, 32768
        T = ref.total_budget(L, N, 0.2)
        R = rng.uniform(0.15, 0.25, L)
        det = ref.allocate_detail(R, T, 1, N)
        if det["cliff_kind"] != "pair" or det["margin"] < 1e-10:
            continue
        x, y = det["cliff_pair"]
        # the bound is tight up to the weight of the two layers themselves in the mean perturbation
        # (2/28 of |q_x - q_y|, itself under a quarter of the shares here): 2 % above it the pair trades
        b, _ = ref.allocate(R * (1.0 + _push_pair(det, R, 1.02 * det["margin"])), T, 1, N)
        diff = b - det["budgets"]
        if np.count_nonzero(diff) > 2:             # another pair sat almost as close to its own cliff
            continue
        want = np.zeros(L, dtype=np.int64)
        want[x], want[y] = -1, 1
        assert np.array_equal(diff, want), (det["cliff_pair"], diff, det["margin"])
        flipped += 1
    assert flipped > 200


def test_margin_clamp_cliff_hand_example():
    # layer 2's share 100 x / (2 + x) is 49.9 for x = 2 * 49.9 / 50.1 (upper bound 50): distance
    # D = 0.1 and weight 0.499, so the share keeps its side while eps < 0.1 / (2 * 0.501 * 49.9 + 0.1)
    x = 2.0 * 49.9 / 50.1
    R = np.array([1.0, 1.0, x])
    det = ref.allocate_detail(R, 100, 1, 50)
    assert det["budgets"].tolist() == [25, 25, 50]     # 25.05, 25.05, 49.9: the left-over row goes to .9
    assert det["cliff_kind"] == "clamp"
    assert math.isclose(det["margin"], 0.1 / (2.0 * (1.0 - 0.499) * 49.9 + 0.1), rel_tol=1e-9)
    # layer 2 up, the others down: the worst direction.  Below the margin the share stays under 50
    # (no layer is pinned, the decision closest to tipping is still this clamp); just above it the
    # share exceeds 50 and the layer is pinned (same vector here: 50 rows either way)
    e = np.array([-1.0, -1.0, 1.0])
    below = ref.allocate_detail(R * (1.0 + 0.99 * det["margin"] * e), 100, 1, 50)
    above = ref.allocate_detail(R * (1.0 + 1.01 * det["margin"] * e), 100, 1, 50)
    assert below["budgets"].tolist() == [25, 25, 50] and below["cliff_kind"] == "clamp"
    assert above["budgets"].tolist() == [25, 25, 50]
    share = lambda Rp: 100.0 * Rp[2] / Rp.sum()
    assert share(R * (1.0 + 0.99 * det["margin"] * e)) < 50.0 < share(R * (1.0 + 1.01 * det["margin"] * e))


def test_integer_crossing_of_a_share_is_not_a_cliff():
    # two layers whose shares sit a hair on either side of an integer give the same budgets
    lo_side = ref.allocate_detail([1.0, 1.0, 2.0 - 1e-9, 4.0], 64, 1, 64)    # share 2 just below 16
    hi_side = ref.allocate_detail([1.0, 1.0, 2.0 + 1e-9, 4.0], 64, 1, 64)    # ... just above 16
    assert lo_side["budgets"].tolist() == hi_side["budgets"].tolist() == [8, 8, 16, 32]
    assert lo_side["margin"] > 1e-3 and hi_side["margin"] > 1e-3


def test_layer_offsets_are_prefix_sums():
    off = ref.layer_offsets(np.array([3, 0, 5]), 4)
    assert off.tolist() == [0, 12, 12, 32]


# ------------------------------------------------------------------- selection
def _brute_force_select(s, k):
    order = sorted(range(len(s)), key=lambda i: (-float(s[i]), i))
    return sorted(order[:k])


def test_select_matches_brute_force_with_ties():
    rng = np.random.default_rng(1)
    for _ in range(200):
        n = int(rng.integers(1, 40))
        k = int(rng.integers(0, n + 1))
        s = rng.integers(0, 6, n).astype(np.float32) * 0.25     # many exact ties
        got = ref.select(s, k)
        assert got.tolist() == _brute_force_select(s, k)
        assert got.dtype == np.int32
        if 0 < k < n:
            dropped = np.setdiff1d(np.arange(n), got)
            assert s[got].min() >= s[dropped].max()


def test_select_special_cases():
    s = np.array([0.5, 0.5, 0.5, 0.5], dtype=np.float32)
    assert ref.select(s, 2).tolist() == [0, 1]                # all equal -> first k
    assert ref.select(s, 4).tolist() == [0, 1, 2, 3]          # k = N keeps all
    assert ref.select(s, 0).tolist() == []
    s = np.array([1.0, 3.0, 2.0, 3.0, 0.0], dtype=np.float32)
    assert ref.select(s, 1).tolist() == [1]                   # tie -> lower index
    assert ref.select(s, 3).tolist() == [1, 2, 3]
    # the decision is taken in fp32: values that differ only beyond fp32 are ties
    s64 = np.array([1.0, 1.0 + 1e-12, 1.0 - 1e-12])
    assert ref.select(s64.astype(np.float32), 1).tolist() == [0]


# ---------------------------------------------------------------------- gather
def test_select_gather_layout_and_bit_copies():
    rng = np.random.default_rng(2)
    L, H, N, d = 3, 2, 20, 8
    K = rng.integers(0, 2 ** 16, (L, H, N, d)).astype(np.uint16)     # arbitrary bf16 bit patterns
    V = rng.integers(0, 2 ** 16, (L, H, N, d)).astype(np.uint16)
    scores = rng.uniform(0, 1, (L, H, N)).astype(np.float32)
    budgets = np.array([4, 1, 7])
    out = ref.select_gather(K, V, scores, budgets)
    assert out["layer_offsets"].tolist() == [0, 8, 10, 24]
    for l in range(L):
        for h in range(H):
            o = out["layer_offsets"][l] + h * budgets[l]
            kept = out["idx"][o:o + budgets[l]]
            assert kept.tolist() == _brute_force_select(scores[l, h], budgets[l])
            assert np.all(np.diff(kept) > 0)
            assert np.array_equal(out["K_out"][o:o + budgets[l]], K[l, h][kept])
            assert np.array_equal(out["V_out"][o:o + budgets[l]], V[l, h][kept])


def test_compress_end_to_end_shapes_and_budget_sum():
    rng = np.random.default_rng(3)
    B, L, H, N, d = 2, 3, 2, 64, 8
    K = rng.standard_normal((B, L, H, N, d)).astype(np.float32)
    V = rng.standard_normal((B, L, H, N, d)).astype(np.float32)
    K[:, 1] *= np.linspace(1.0, 0.01, N)[None, None, :, None]       # layer 1 smoother along tokens
    r, T = ref.cutoff_r(N, 0.1), ref.total_budget(L, N, 0.25)
    out = ref.compress(K, V, "f32", r, T, route="definition")
    assert out["budgets"].shape == (B, L) and np.all(out["budgets"].sum(axis=1) == T)
    assert out["idx"].shape == (B, H * T) and out["K_out"].shape == (B, H * T, d)
    assert out["scores"].dtype == np.float32


# ------------------------------------------------------------ layer-shared mode
def test_layer_score_is_row_wide_mse_and_shared_selection():
    # the MSE of a token over the whole H*d wide row of a layer = mean of the per-head MSEs
    rng = np.random.default_rng(7)
    H, N, d, r = 3, 96, 8, 9
    K = rng.standard_normal((1, H, N, d)).astype(np.float32)
    V = rng.standard_normal((1, H, N, d)).astype(np.float32)
    K[0, 1, 40] += 6.0
    per_head = ref.score(K, V, "f32", r, "definition")["score"][0]                  # [H, N]
    wide_k = np.concatenate([K[0, h] for h in range(H)], axis=1).astype(np.float64)  # [N, H*d]
    wide_v = np.concatenate([V[0, h] for h in range(H)], axis=1).astype(np.float64)
    dk, dv = ref.score_unit(wide_k, wide_v, r, "definition")
    assert np.allclose(dk + dv, per_head.mean(axis=0), rtol=1e-12)
    ls = ref.layer_score(per_head.astype(np.float32))
    assert ls.dtype == np.float32 and np.allclose(ls, dk + dv, rtol=1e-6)
    out = ref.select_gather(K[0][None], V[0][None], per_head.astype(np.float32)[None], np.array([10]),
                            shared=True)
    want = sorted(np.argsort(-(dk + dv), kind="stable")[:10].tolist())
    for h in range(H):
        assert out["idx"][h * 10:(h + 1) * 10].tolist() == want
        assert np.array_equal(out["K_out"][h * 10:(h + 1) * 10], K[0, h][want])
    assert 40 in want
    # with one head the shared mode is the per-head mode
    a = ref.select_gather(K[:, :1], V[:, :1], per_head[None, :1].astype(np.float32), np.array([7]))
    b = ref.select_gather(K[:, :1], V[:, :1], per_head[None, :1].astype(np.float32), np.array([7]), shared=True)
    assert np.array_equal(a["idx"], b["idx"])


def test_scatter_paged_round_trip():
    rng = np.random.default_rng(9)
    L, H, d, page = 2, 2, 4, 3
    budgets = np.array([5, 2])
    rows = H * int(budgets.sum())
    packed = rng.integers(1, 1000, (rows, d)).astype(np.float32)
    pages_per_unit = 2
    table = rng.permutation(L * H * pages_per_unit).reshape(L, H, pages_per_unit).astype(np.int32)
    cache = np.zeros((L * H * pages_per_unit, page, d), dtype=np.float32)
    ref.scatter_paged(packed, budgets, H, table, page, cache)
    off = ref.layer_offsets(budgets, H)
    for l in range(L):
        for h in range(H):
            o = off[l] + h * budgets[l]
            back = np.concatenate([cache[table[l, h, p]] for p in range(pages_per_unit)])[:budgets[l]]
            assert np.array_equal(back, packed[o:o + budgets[l]])
    assert np.count_nonzero(cache.any(axis=2)) == rows            # nothing else was touched


def test_decode_attention_special_cases():
    rng = np.random.default_rng(11)
    L, H, G, d = 2, 2, 2, 8
    budgets = np.array([3, 1])
    rows = H * int(budgets.sum())
    Kr = rng.standard_normal((rows, d)).astype(np.float32)
    Vr = rng.standard_normal((rows, d)).astype(np.float32)
    Q = rng.standard_normal((L, H * G, d)).astype(np.float32)
    out = ref.decode_attention(Q, Kr, Vr, "f32", budgets, H, 0.5)
    # a unit with one row returns that row of V whatever q is (layer 1: rows 6 and 7)
    assert np.allclose(out[1, 0], Vr[6]) and np.allclose(out[1, 1], Vr[6]) and np.allclose(out[1, 2], Vr[7])
    # zero query -> uniform weights -> mean of the unit's V rows
    out0 = ref.decode_attention(np.zeros_like(Q), Kr, Vr, "f32", budgets, H, 0.5)
    assert np.allclose(out0[0, 0], Vr[0:3].mean(axis=0)) and np.allclose(out0[0, 3], Vr[3:6].mean(axis=0))
    # a very large logit on one row selects it; weights are invariant to a shift of all logits
    Kr2 = Kr.copy()
    Kr2[1] = 50.0 * Q[0, 0] / np.dot(Q[0, 0], Q[0, 0])
    sel = ref.decode_attention(Q, Kr2, Vr, "f32", budgets, H, 10.0)
    assert np.allclose(sel[0, 0], Vr[1], atol=1e-6)
    # brute force for one head
    s = (Kr[0:3].astype(np.float64) @ Q[0, 1].astype(np.float64)) * 0.5
    w = np.exp(s) / np.exp(s).sum()
    assert np.allclose(out[0, 1], w @ Vr[0:3].astype(np.float64))


def test_decode_attention_paged_equals_packed_after_scatter():
    """Scattering the packed rows into pages and attending through the block table is the same as
    attending over the packed rows; rows of a page that was never mapped are left out."""
    rng = np.random.default_rng(11)
    L, H, Hq, d, page = 3, 2, 6, 8, 4
    budgets = np.array([5, 0, 9])
    rows = int(ref.layer_offsets(budgets, H)[-1])
    Kr, Vr = rng.standard_normal((rows, d)).astype(np.float32), rng.standard_normal((rows, d)).astype(np.float32)
    Q = rng.standard_normal((L, Hq, d)).astype(np.float32)
    max_pages = 3
    table = rng.permutation(L * H * max_pages).reshape(L, H, max_pages).astype(np.int32)
    n_pages = L * H * max_pages
    Kc = ref.scatter_paged(Kr, budgets, H, table, page, np.zeros((n_pages, page, d), np.float32))
    Vc = ref.scatter_paged(Vr, budgets, H, table, page, np.zeros((n_pages, page, d), np.float32))
    want = ref.decode_attention(Q, Kr, Vr, "f32", budgets, H, 0.3)
    got = ref.decode_attention_paged(Q, Kc, Vc, "f32", budgets, H, table, page, 0.3)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    # unmap the last page of unit (2, 1): its rows 8.. drop out, i.e. the unit attends to 8 rows only
    table2 = table.copy()
    table2[2, 1, 2] = -1
    got2 = ref.decode_attention_paged(Q, Kc, Vc, "f32", budgets, H, table2, page, 0.3)
    off = ref.layer_offsets(budgets, H)
    o = int(off[2]) + 1 * 9
    k8, v8 = Kr[o:o + 8].astype(np.float64), Vr[o:o + 8].astype(np.float64)
    for g in range(3, 6):
        s_ = (k8 @ Q[2, g].astype(np.float64)) * 0.3
        p_ = np.exp(s_ - s_.max())
        np.testing.assert_allclose(got2[2, g], (p_ / p_.sum()) @ v8, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(got2[:2], want[:2], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(got2[2, :3], want[2, :3], rtol=1e-12, atol=1e-12)
