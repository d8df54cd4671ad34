"""Pins for the oracle's transform, low-pass and deviation score (Eq. 6-10).

None of these re-types the oracle's own formula: each compares it with a
library routine, a closed form, an invariant or a special case.
"""
import math

import numpy as np
import pytest
import scipy.fft

from oracle import flashcache_ref as ref


def _rand(n, d, seed=0):
    return np.random.default_rng(seed).standard_normal((n, d))


# ---------------------------------------------------------------- basis (Eq. 7)
@pytest.mark.parametrize("n", [1, 2, 7, 64, 200, 256])
def test_basis_is_orthonormal(n):
    m = ref.dct_basis(n, n)
    assert np.allclose(m.T @ m, np.eye(n), atol=1e-12)
    assert np.allclose(m @ m.T, np.eye(n), atol=1e-12)


@pytest.mark.parametrize("n", [5, 16, 33, 128])
def test_basis_equals_library_dct2_ortho(n):
    # column i of the library transform of the identity = coefficients of e_i
    lib = scipy.fft.dct(np.eye(n), type=2, norm="ortho", axis=0)      # lib[m, i]
    assert np.allclose(ref.dct_basis(n, n).T, lib, atol=1e-13)


def test_basis_n4_closed_form_radicals():
    # N=4: alpha*phi are 1/2, and cos(pi/8), cos(3pi/8) over sqrt 2, with known signs
    c1 = math.sqrt(2.0 + math.sqrt(2.0)) / 2.0 / math.sqrt(2.0)
    c3 = math.sqrt(2.0 - math.sqrt(2.0)) / 2.0 / math.sqrt(2.0)
    want = np.array([[0.5, 0.5, 0.5, 0.5],
                     [c1, c3, -c3, -c1],
                     [0.5, -0.5, -0.5, 0.5],
                     [c3, -c1, c1, -c3]])
    assert np.allclose(ref.dct_basis(4, 4).T, want, atol=1e-15)


def test_basis_mirror_symmetry_and_large_index_reduction():
    n = 32768
    m = ref.dct_basis(n, 1639)
    # phi(m, N-1-i) = (-1)^m phi(m, i)
    sign = np.where(np.arange(1639) % 2 == 0, 1.0, -1.0)
    assert np.allclose(m[::-1], m * sign[None, :], atol=1e-15)
    # unit-norm columns even at the largest arguments
    assert np.allclose(np.sum(m * m, axis=0), 1.0, atol=1e-12)


# ------------------------------------------------- fast route == explicit sums
@pytest.mark.parametrize("n,r", [(8, 3), (17, 5), (64, 7), (512, 52), (100, 100), (33, 1)])
def test_fast_route_equals_definition(n, r):
    x = _rand(n, 6, seed=n)
    assert np.allclose(ref.base_fast(x.copy(), r), ref.base_definition(x, r), atol=1e-10)


def test_coefficients_equal_library():
    x = _rand(96, 5, 3)
    assert np.allclose(ref.coefficients_definition(x),
                       scipy.fft.dct(x, type=2, norm="ortho", axis=0), atol=1e-12)


# -------------------------------------------------------- mask boundary (Eq. 8)
def test_cutoff_r_values():
    assert ref.cutoff_r(512, 0.1) == 52
    assert ref.cutoff_r(4096, 0.1) == 410
    assert ref.cutoff_r(8192, 0.1) == 820
    assert ref.cutoff_r(32768, 0.05) == 1639
    assert ref.cutoff_r(16384, 0.1) == 1639
    assert ref.cutoff_r(10, 0.0) == 1          # omega = 0 keeps mode 0
    assert ref.cutoff_r(10, 1.0) == 10         # never more than N
    assert ref.cutoff_r(10, 0.5) == 6          # modes 0..5 inclusive


def test_total_budget_values():
    assert ref.total_budget(1, 512, 0.2) == 102
    assert ref.total_budget(4, 4096, 0.2) == 3276
    assert ref.total_budget(28, 8192, 0.2) == 45875
    assert ref.total_budget(28, 32768, 0.2) == 183500
    assert ref.total_budget(28, 16384, 0.1) == 45875
    assert ref.total_budget(4, 100, 0.0) == 4
    assert ref.total_budget(4, 100, 2.0) == 400


@pytest.mark.parametrize("route", ["definition", "fast"])
def test_keep_all_modes_gives_zero_scores(route):
    k, v = _rand(40, 8, 1), _rand(40, 8, 2)
    dk, dv = ref.score_unit(k, v, 40, route)
    assert np.max(np.abs(dk)) < 1e-24 * 1e6 and np.max(np.abs(dv)) < 1e-18


@pytest.mark.parametrize("route", ["definition", "fast"])
def test_keep_only_mode0_gives_deviation_from_column_mean(route):
    k, v = _rand(50, 12, 5), 3.0 + _rand(50, 12, 6)
    dk, dv = ref.score_unit(k, v, 1, route)
    assert np.allclose(dk, np.mean((k - k.mean(axis=0)) ** 2, axis=1), atol=1e-12)
    assert np.allclose(dv, np.mean((v - v.mean(axis=0)) ** 2, axis=1), atol=1e-12)


def test_adding_one_mode_removes_exactly_its_energy():
    n, d, r = 64, 4, 9
    x = _rand(n, d, 8)
    c = scipy.fft.dct(x, type=2, norm="ortho", axis=0)
    e_r = d * ref.deviation(x, ref.base_definition(x, r)).sum()
    e_r1 = d * ref.deviation(x, ref.base_definition(x, r + 1)).sum()
    assert math.isclose(e_r - e_r1, float(np.sum(c[r] ** 2)), rel_tol=1e-10)


# ------------------------------------------------------------- scoring (Eq. 10)
def _dirichlet(theta, r):
    """sum_{m=-(r-1)}^{r-1} exp(i m theta) = sin((r-1/2) theta)/sin(theta/2)."""
    theta = np.asarray(theta, dtype=np.float64)
    out = np.full(theta.shape, 2.0 * r - 1.0)
    nz = np.abs(np.sin(theta / 2.0)) > 1e-14
    out[nz] = np.sin((r - 0.5) * theta[nz]) / np.sin(theta[nz] / 2.0)
    return out


@pytest.mark.parametrize("n,r,x0", [(64, 7, 10), (200, 20, 0), (128, 13, 127)])
def test_single_spike_closed_form(n, r, x0):
    # one spike A at token x0 on a zero background: base[x] = P[x, x0] * A where the
    # low-pass projector is a sum of two Dirichlet kernels (symmetric extension):
    # P[x, y] = (D((x-y) pi/N) + D((x+y+1) pi/N)) / (2N)
    d = 5
    a = np.array([1.0, -2.0, 0.5, 3.0, -1.5])
    k = np.zeros((n, d))
    k[x0] = a
    v = np.zeros((n, d))
    x = np.arange(n)
    p = (_dirichlet((x - x0) * np.pi / n, r) + _dirichlet((x + x0 + 1) * np.pi / n, r)) / (2.0 * n)
    want = np.mean(a * a) * ((x == x0).astype(np.float64) - p) ** 2
    for route in ("definition", "fast"):
        dk, dv = ref.score_unit(k, v, r, route)
        assert np.allclose(dk, want, atol=1e-13)
        assert np.max(np.abs(dv)) == 0.0


@pytest.mark.parametrize("route", ["definition", "fast"])
def test_pure_low_frequency_input_scores_zero(route):
    n, d, r = 512, 16, 52
    rng = np.random.default_rng(11)
    t = np.arange(n) + 0.5
    x = sum(rng.standard_normal() * np.cos(np.pi * t * j / n)[:, None] * rng.standard_normal(d)[None, :]
            for j in range(8))
    dk, dv = ref.score_unit(x, 2.0 * x, r, route)
    power = np.mean(x * x)
    assert np.max(dk) <= 1e-20 * power * n and np.max(dv) <= 1e-20 * power * n * 4


def test_injected_outlier_ranks_first():
    n, d, r = 256, 32, 26
    rng = np.random.default_rng(12)
    t = np.arange(n) + 0.5
    smooth = np.cos(np.pi * t * 3 / n)[:, None] * rng.standard_normal(d)[None, :]
    k = smooth + 0.1 * rng.standard_normal((n, d))
    v = smooth + 0.1 * rng.standard_normal((n, d))
    k[77] += 5.0 * rng.standard_normal(d)
    dk, dv = ref.score_unit(k, v, r, "definition")
    assert int(np.argmax(dk + dv)) == 77
    kept = ref.select((dk + dv).astype(np.float32), 1)
    assert kept.tolist() == [77]


def test_scaling_idempotence_reversal_permutation():
    n, d, r = 96, 10, 11
    k, v = _rand(n, d, 20), _rand(n, d, 21)
    dk, dv = ref.score_unit(k, v, r, "definition")
    # scaling the input by a scales scores by a^2
    dk2, dv2 = ref.score_unit(-3.0 * k, 0.5 * v, r, "definition")
    assert np.allclose(dk2, 9.0 * dk, rtol=1e-12) and np.allclose(dv2, 0.25 * dv, rtol=1e-12)
    # the base is a projection: scoring the base itself gives zero
    kb = ref.base_definition(k, r)
    dkb, _ = ref.score_unit(kb, v, r, "definition")
    assert np.max(dkb) < 1e-26 * n
    # reversing the token order reverses the scores
    dkr, dvr = ref.score_unit(k[::-1].copy(), v[::-1].copy(), r, "definition")
    assert np.allclose(dkr, dk[::-1], atol=1e-13) and np.allclose(dvr, dv[::-1], atol=1e-13)
    # permuting feature columns changes nothing
    perm = np.random.default_rng(0).permutation(d)
    dkp, _ = ref.score_unit(k[:, perm], v, r, "definition")
    assert np.allclose(dkp, dk, atol=1e-13)


def test_units_are_independent_and_score_is_sum():
    n, d, r = 64, 8, 7
    K = np.random.default_rng(30).standard_normal((1, 2, 3, n, d)).astype(np.float32)
    V = np.random.default_rng(31).standard_normal((1, 2, 3, n, d)).astype(np.float32)
    a = ref.score(K, V, "f32", r, "definition")
    K2 = K.copy()
    K2[0, 1, 2] *= 7.0                                   # touch one unit only
    b = ref.score(K2, V, "f32", r, "definition")
    changed = np.zeros((1, 2, 3), dtype=bool)
    changed[0, 1, 2] = True
    assert np.array_equal(a["score"][~changed], b["score"][~changed])
    assert not np.allclose(a["score"][changed], b["score"][changed])
    assert np.allclose(a["score"], a["dev_k"] + a["dev_v"])


# ----------------------------------------------------- energies (Eq. 11-12)
def test_parseval_links_scores_to_spectrum_tail():
    n, d, r = 160, 12, 17
    K = _rand(n, d, 40).astype(np.float32)[None]
    V = (2.0 * _rand(n, d, 41)).astype(np.float32)[None]
    out = ref.score(K, V, "f32", r, "definition")
    for t, X in enumerate((K[0], V[0])):
        c = scipy.fft.dct(X.astype(np.float64), type=2, norm="ortho", axis=0)
        p = np.sum(c * c, axis=1)                                  # P[m] = |C[m]|^2
        assert math.isclose(out["energy"][0, t], p[r:].sum(), rel_tol=1e-11)
        assert math.isclose(out["energy"][0, 2 + t], p.sum(), rel_tol=1e-12)


def test_layer_ratio_hand_example_and_bounds():
    # two heads: K high-pass energies 1 and 3 of totals 10 and 30 -> 4/40; V: 2+2 of 8+8 -> 4/16
    e = np.array([[[1.0, 2.0, 10.0, 8.0], [3.0, 2.0, 30.0, 8.0]],
                  [[0.0, 0.0, 0.0, 0.0], [0.0, 0.0, 0.0, 0.0]]])
    R = ref.layer_ratios(e)
    assert R[0] == 4.0 / 40.0 + 4.0 / 16.0
    assert R[1] == 0.0
    K = _rand(64, 4, 50).astype(np.float32)[None, None]
    out = ref.score(K, K, "f32", 5, "fast")
    R = ref.layer_ratios(out["energy"])
    assert 0.0 <= R[0] <= 2.0


def test_white_noise_ratio_is_one_minus_r_over_n():
    n, d, r = 1024, 64, 103
    K = (0.3 * _rand(n, d, 60)).astype(np.float32)[None, None]
    V = (5.0 * _rand(n, d, 61)).astype(np.float32)[None, None]
    R = ref.layer_ratios(ref.score(K, V, "f32", r, "fast")["energy"])
    assert abs(R[0] - 2.0 * (1.0 - r / n)) < 0.02


def test_bf16_widening_is_exact():
    bits = np.array([0x3F80, 0xC000, 0x3DCD, 0x0000, 0x7F7F], dtype=np.uint16)
    got = ref.widen(bits, "bf16")
    want = np.array([1.0, -2.0, 0.10009765625, 0.0, 3.3895313892515355e38])
    assert np.array_equal(got, want)


def test_spectrum_energies_split_the_total_at_the_cutoff():
    n, d, r = 120, 6, 13
    x = _rand(n, d, 70)
    lo, hi = ref.spectrum_energies(x, r)
    assert math.isclose(lo + hi, float(np.sum(x * x)), rel_tol=1e-12)
    assert math.isclose(hi, d * ref.deviation(x, ref.base_definition(x, r)).sum(), rel_tol=1e-10)
    lo_all, hi_all = ref.spectrum_energies(x, n)
    assert hi_all == 0.0 and math.isclose(lo_all, float(np.sum(x * x)), rel_tol=1e-12)
