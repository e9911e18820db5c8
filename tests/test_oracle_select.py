"""Pins for the oracle's selection (paper Sec. 3.3, probability-based selection function)."""
import itertools
import math
import os

import numpy as np
import pytest
from scipy import stats

import oracle


def _read_kat(golden_dir):
    rows = []
    for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(t, 16) for t in line.split()]
        rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def _philox_bigint(ctr, key):
    """Independent statement of the published round function with Python integers."""
    c = list(ctr); k = list(key)
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]; p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_philox_known_answers(golden_dir):
    for ctr, key, out in _read_kat(golden_dir):
        assert oracle.philox4x32_10(ctr, key).tolist() == out


def test_philox_against_bigint_round_function():
    rng = np.random.default_rng(0)
    for _ in range(200):
        ctr = rng.integers(0, 2 ** 32, size=4).tolist(); key = rng.integers(0, 2 ** 32, size=2).tolist()
        assert oracle.philox4x32_10(ctr, key).tolist() == _philox_bigint(ctr, key)


def test_uniform_is_top_53_bits_of_words_1_and_0():
    seed, cycle, t = 2021, (5 << 32) | 7, 3
    o = _philox_bigint([7, 5, 3, 0], [2021, 0])
    u = oracle.uniform(seed, cycle, t)
    assert u == ((o[1] << 32 | o[0]) >> 11) * 2.0 ** -53 and 0.0 <= u < 1.0
    us = np.array([oracle.uniform(9, c, 0) for c in range(20000)])
    assert abs(us.mean() - 0.5) < 0.01 and abs(us.var() - 1 / 12) < 0.005


def test_deterministic_exp_is_exp():
    xs = np.concatenate([np.linspace(-690, 0, 5001), -np.arange(0, 200) ** 2 / 32.0])
    xs = xs[xs >= -690]
    for x in xs:
        a, b = oracle.exp_det(x), math.exp(x)
        assert abs(a - b) <= 4 * np.spacing(b), x
    assert oracle.exp_det(0.0) == 1.0 and oracle.exp_det(-690.0) > 0.0


@pytest.mark.parametrize("v,mu", [([1, 2, 3, 4], 3.25), ([3, 3, 1, 1], 3.0), ([4, 2, 2, 1], 2.5),
                                  ([1, 1, 2, 2, 3, 3, 4, 4], 3.25), ([7], 7.0), ([2, 9], 7.25)])
def test_third_quartile(v, mu):
    assert oracle.select(v, 1, 0, 0)[3] == mu == np.percentile(v, 75)


def test_third_quartile_random_against_numpy():
    rng = np.random.default_rng(4)
    for _ in range(100):
        v = rng.integers(0, 51, size=rng.integers(1, 70))
        assert oracle.select(v, 1, 0, 0)[3] == np.percentile(v, 75)


@pytest.mark.parametrize("v", [[1, 2, 3, 4], [3, 3, 1, 1], [4, 2, 2, 1], [1, 1, 2, 2, 3, 3, 4, 4], [5, 5, 5]])
def test_probabilities_are_the_unit_variance_gaussian_about_q3(v):
    P = oracle.probabilities(v)
    pdf = stats.norm.pdf(np.asarray(v, dtype=float), loc=np.percentile(v, 75), scale=1.0)
    assert np.allclose(P, pdf / pdf.sum(), rtol=1e-13, atol=0)
    assert abs(P.sum() - 1.0) < 1e-15


def test_probability_shape_claims_of_sec_3_3():
    # newer (larger version) => more likely, below the quartile; medial versions beat the latest ones
    P = oracle.probabilities([4, 2, 2, 1])
    assert P[1] == P[2] > P[0] and P[1] > P[3] and abs(P[0] - P[3]) < 1e-15      # symmetric about mu = 2.5
    P = oracle.probabilities([1, 2, 3, 4])
    assert P[0] < P[1] < P[2] and P[2] > P[3]
    # Sec. 4.2 bounds the chance of picking a slow device of [3,3,1,1] by 1/8
    P = oracle.probabilities([3, 3, 1, 1])
    assert P[2] <= 1 / 8 and P[3] <= 1 / 8
    assert np.allclose(oracle.probabilities([6, 6, 6, 6]), 0.25)


def test_far_versions_keep_a_nonzero_probability():
    f = oracle.select([0, 50, 50, 50, 50], 1, 0, 0)[2]
    assert f[0] == oracle.exp_det(-690.0) > 0.0


def _exact_set_probabilities(P, n_select):
    N = len(P)
    out = {}
    for perm in itertools.permutations(range(N), n_select):
        p, rest = 1.0, 1.0
        for k in perm:
            p *= P[k] / rest
            rest -= P[k]
        key = tuple(sorted(perm))
        out[key] = out.get(key, 0.0) + p
    return out


@pytest.mark.parametrize("v,n_select", [([1, 2, 3, 4], 2), ([4, 2, 2, 1], 2), ([1, 2, 3, 4, 2], 3)])
def test_sampler_matches_brute_force_enumeration(v, n_select):
    P = oracle.probabilities(v)
    exact = _exact_set_probabilities(P, n_select)
    assert abs(sum(exact.values()) - 1.0) < 1e-12
    draws = 200000
    counts = dict.fromkeys(exact, 0)
    first = np.zeros(len(v))
    for c in range(draws):
        sel, flag, _, _ = oracle.select(v, n_select, 2021, c)
        assert len(set(sel.tolist())) == n_select and flag.sum() == n_select
        counts[tuple(sorted(sel.tolist()))] += 1
        first[sel[0]] += 1
    chi2 = sum((counts[k] - draws * p) ** 2 / (draws * p) for k, p in exact.items())
    assert chi2 < stats.chi2.ppf(0.9999, len(exact) - 1), (chi2, counts)
    chi2_first = ((first - draws * P) ** 2 / (draws * P)).sum()
    assert chi2_first < stats.chi2.ppf(0.9999, len(v) - 1)


def test_first_draw_is_inverse_cdf_of_the_uniform():
    v = [1, 2, 3, 4]
    f = oracle.select(v, 1, 0, 0)[2]
    for c in range(500):
        u = oracle.uniform(77, c, 0)
        k = int(np.searchsorted(np.cumsum(f), u * f.sum(), side="right"))
        assert oracle.select(v, 1, 77, c)[0][0] == min(k, 3)


def test_select_all_and_availability_mask():
    v = [3, 1, 4, 1, 5, 9, 2, 6]
    sel, flag, _, _ = oracle.select(v, 8, 1, 0)
    assert sorted(sel.tolist()) == list(range(8)) and flag.all()
    avail = np.array([1, 0, 1, 1, 0, 1, 1, 1], dtype=np.uint8)
    for c in range(300):
        sel, flag, f, mu = oracle.select(v, 3, 1, c, avail)
        assert not flag[1] and not flag[4] and f[1] == 0 and f[4] == 0
        assert mu == np.percentile(np.asarray(v)[avail.astype(bool)], 75)
    with pytest.raises(ValueError):
        oracle.select(v, 7, 1, 0, avail)


def test_aggregation_weights_sum_to_one():
    sel, flag, f, _ = oracle.select([1, 2, 3, 4, 4, 2], 3, 5, 11)
    for mode in (0, 1):
        a = oracle.aggregation_weights(flag, f, mode)
        assert abs(a.sum() - 1.0) < 1e-15 and np.all(a[flag == 0] == 0)
    assert np.all(oracle.aggregation_weights(flag, f, 0)[flag == 1] == 1 / 3)


def test_real_valued_versions_same_rule():
    # Sec. 3.2 forecasts are real numbers; Sec. 3.3's rule only uses v - Q3(v).  Integer versions given as floats select
    # the same devices; adding one constant to every version changes nothing; and the probabilities are the unit-variance
    # Gaussian about the interpolated quartile, written out by hand for one case.
    v_int = np.array([4, 2, 2, 1, 3, 3, 1, 5])
    for cycle in range(20):
        a = oracle.select(v_int, 3, 7, cycle)
        b = oracle.select(v_int.astype(np.float64), 3, 7, cycle)
        c = oracle.select(v_int.astype(np.float64) + 0.5, 3, 7, cycle)       # exact shift: quartile moves with it
        assert a[0].tolist() == b[0].tolist() == c[0].tolist()
        assert np.array_equal(a[2], b[2]) and np.array_equal(a[2], c[2])
    v = np.array([0.5, 1.25, 3.0, 2.5])
    sel, flag, f, mu = oracle.select(v, 2, 7, 0)
    # sorted 0.5 1.25 2.5 3.0; position 0.75 * 3 = 2.25 -> 2.5 + 0.25 * 0.5
    assert mu == 2.625
    want = np.exp(-0.5 * (v - 2.625) ** 2)
    assert np.abs(f - want).max() < 1e-15
    assert np.abs(oracle.probabilities(v) - want / want.sum()).max() < 1e-15
