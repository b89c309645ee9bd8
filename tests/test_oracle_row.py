"""Pins for the oracle's per-row definition (softmax, entropy of Eq. 2, top-K of Sec. 4.2.2):
closed forms, invariants and library routines.  CPU only."""
import math

import numpy as np
import pytest
from scipy.special import softmax
from scipy.stats import entropy

from oracle import ref_entropy_top_m, ref_row


def _bf16_bits(x32):
    """fp32 -> bf16 bits, round to nearest even (numpy-only, for building test rows)."""
    u = np.asarray(x32, np.float32).view(np.uint32).astype(np.uint64)
    r = ((u >> 16) & 1) + 0x7FFF
    return ((u + r) >> 16).astype(np.uint16)


def _widen(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def test_softmax_sums_to_one_and_matches_library():
    rng = np.random.default_rng(1)
    for V in (7, 64, 1000, 5003):
        x = (3.0 * rng.standard_normal(V)).astype(np.float32)
        r = ref_row(x, V)                       # K = V returns every probability
        assert not r["bad"]
        assert abs(r["p"].sum() - 1.0) < 1e-12
        p_lib = softmax(x.astype(np.float64))
        got = np.zeros(V)
        got[r["ids"]] = r["p"]
        np.testing.assert_allclose(got, p_lib, rtol=1e-12, atol=0)
        assert r["m"] == float(x.max())
        assert abs(r["H"] - entropy(p_lib)) < 1e-12


def test_entropy_two_formulas_agree_and_bounds():
    rng = np.random.default_rng(2)
    for V in (2, 33, 4096):
        x = (5.0 * rng.standard_normal(V)).astype(np.float32)
        r = ref_row(x, V)
        p = r["p"]
        H2 = -np.sum(p[p > 0] * np.log(p[p > 0]))     # -sum p ln p from the returned p
        assert abs(r["H"] - H2) < 1e-12
        assert abs((math.log(r["Z"]) - r["S"] / r["Z"]) - r["H"]) < 1e-15
        assert -1e-15 <= r["H"] <= math.log(V) + 1e-12


def test_shift_invariance_exact_shift():
    rng = np.random.default_rng(3)
    x = (rng.integers(-4000, 4000, 777) / 256.0).astype(np.float32)   # multiples of 2^-8: x+8 is exact
    a = ref_row(x, 10)
    b = ref_row((x + np.float32(8.0)).astype(np.float32), 10)
    np.testing.assert_array_equal(a["ids"], b["ids"])
    np.testing.assert_allclose(a["p"], b["p"], rtol=1e-14)
    assert abs(a["H"] - b["H"]) < 1e-13
    assert b["m"] == a["m"] + 8.0


def test_uniform_row():
    for V in (1, 5, 32000):
        r = ref_row(np.full(V, 1.25, np.float32), min(V, 10))
        assert abs(r["H"] - math.log(V)) < 1e-12
        np.testing.assert_allclose(r["p"], 1.0 / V, rtol=1e-13)
        np.testing.assert_array_equal(r["ids"], np.arange(min(V, 10)))   # ties -> lower id first


def test_one_hot_and_two_valued_closed_form():
    V = 1000
    x = np.zeros(V, np.float32)
    x[123] = 80.0
    r = ref_row(x, 3)
    assert r["ids"][0] == 123 and list(r["ids"][1:]) == [0, 1]
    assert 0 <= r["H"] < 1e-25                  # ~ 999 * 81 * e^-80
    # a tokens at value u, V-a tokens at 0
    for a, u in ((1, 3.0), (10, 1.5), (999, -2.0)):
        x = np.zeros(V, np.float32)
        x[:a] = u
        r = ref_row(x, 1)
        Z = a * math.exp(u) + (V - a)
        p1, p0 = math.exp(u) / Z, 1.0 / Z
        H = -(a * p1 * math.log(p1) + (V - a) * p0 * math.log(p0))
        assert abs(r["H"] - H) < 1e-12
        assert abs(r["p"][0] - max(p1, p0)) < 1e-15


def test_noise_free_zipf_closed_form():
    # x_t = -s ln(rank): p_r = r^-s / H_{V,s};  H = s * sum(r^-s ln r)/H_{V,s} + ln H_{V,s}
    V, s = 32000, 1.1
    ranks = np.arange(1, V + 1, dtype=np.float64)
    x = (-s * np.log(ranks)).astype(np.float32)
    r = ref_row(x, 5)
    w = ranks ** (-s)
    Hvs = w.sum()
    H = s * np.sum(w * np.log(ranks)) / Hvs + math.log(Hvs)
    assert abs(r["H"] - H) < 5e-6            # x is rounded to fp32 (relative 6e-8 of ~11)
    np.testing.assert_allclose(r["p"], w[:5] / Hvs, rtol=2e-6)
    np.testing.assert_array_equal(r["ids"], np.arange(5))


def test_topk_equals_library_sort_with_ties():
    rng = np.random.default_rng(5)
    for V, K in ((50, 50), (1000, 16), (4099, 32)):
        x = _widen(_bf16_bits(2.0 * rng.standard_normal(V)))          # bf16 grid: many exact ties
        r = ref_row(x, K)
        order = np.lexsort((np.arange(V), -x.astype(np.float64)))[:K]  # (value desc, id asc)
        np.testing.assert_array_equal(r["ids"], order)
        np.testing.assert_array_equal(r["logits"], x[order].astype(np.float64))
    assert len(set(x.tolist())) < V


def test_topk_permutation_equivariance():
    rng = np.random.default_rng(6)
    V, K = 500, 8
    x = rng.permutation(V).astype(np.float32)          # distinct values
    perm = rng.permutation(V)
    a = ref_row(x, K)
    b = ref_row(x[perm], K)                            # position i of b holds token perm[i] of a
    np.testing.assert_array_equal(perm[b["ids"]], a["ids"])
    np.testing.assert_allclose(a["p"], b["p"], rtol=1e-9)   # summation order differs


def test_signed_zero_and_minus_inf():
    x = np.array([-0.0, 0.0, -np.inf, 0.0, -1.0], np.float32)
    r = ref_row(x, 5)
    np.testing.assert_array_equal(r["ids"], [0, 1, 3, 4, 2])     # -0 == +0 ties by id; -inf last
    assert r["p"][4] == 0.0
    assert abs(r["p"].sum() - 1) < 1e-15
    Z = 3 + math.exp(-1)
    assert abs(r["Z"] - Z) < 1e-15


@pytest.mark.parametrize("bad", ["nan", "inf", "allneg"])
def test_bad_rows(bad):
    x = np.zeros(16, np.float32)
    if bad == "nan":
        x[3] = np.nan
    elif bad == "inf":
        x[3] = np.inf
    else:
        x[:] = -np.inf
    assert ref_row(x, 4)["bad"]


def test_bf16_is_exact_widening():
    rng = np.random.default_rng(7)
    bits = _bf16_bits(4.0 * rng.standard_normal(3000))
    a = ref_row(bits, 12)
    b = ref_row(_widen(bits), 12)
    np.testing.assert_array_equal(a["ids"], b["ids"])
    assert a["H"] == b["H"] and a["Z"] == b["Z"] and a["m"] == b["m"]
    np.testing.assert_array_equal(a["p"], b["p"])


def test_entropy_top_m_variant():
    # Eq. 2, second line: sum over the M most probable tokens of the full softmax's p
    rng = np.random.default_rng(8)
    V = 5000
    x = (3.0 * rng.standard_normal(V) - 1.1 * np.log(rng.permutation(V) + 1.0)).astype(np.float32)
    p = np.sort(softmax(x.astype(np.float64)))[::-1]
    full = ref_row(x, 1)["H"]
    prev = 0.0
    for M in (1, 10, 100, 1000, V):
        HM = ref_entropy_top_m(x, M)
        assert abs(HM - (-np.sum(p[:M] * np.log(p[:M])))) < 1e-12
        assert prev - 1e-15 <= HM <= full + 1e-12        # non-decreasing in M, bounded by full
        prev = HM
    assert abs(ref_entropy_top_m(x, V) - full) < 1e-12
