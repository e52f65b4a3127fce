"""Pins of the oracle's randomness, sampling distribution and decisions (CPU only).

Each test checks the oracle against something fixed outside it: published
known-answer vectors, double-precision library arithmetic, exhaustive
enumeration, or the statements of the paper's appendix (Theorem 1).
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# ---------------------------------------------------------------- Philox
def test_philox_known_answers(oracle):
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        assert oracle.philox(v[:4], v[4:6]) == v[6:]
        n += 1
    assert n == 3


def test_philox_uniformity(oracle):
    # 16 equiprobable cells on each of the 4 output words over 50k counters
    counts = np.zeros((4, 16), dtype=np.int64)
    for i in range(50000):
        w = oracle.philox([i, 3, 1, 0], [12345, 0])
        for j in range(4):
            counts[j, w[j] >> 28] += 1
    for j in range(4):
        assert stats.chisquare(counts[j]).pvalue > 1e-3


# ---------------------------------------------------------------- EXP
def test_exp_matches_double_exponential(oracle):
    xs = np.concatenate([-np.random.default_rng(0).uniform(0, 60, 20000), [0.0, -1e-8, -59.999, -0.34657, -0.34658]])
    worst = 0.0
    for x in xs.astype(np.float32):
        got = oracle.exp_neg(float(x))
        want = math.exp(float(x))
        worst = max(worst, abs(got - want) / want)
    assert worst < 4e-7
    assert oracle.exp_neg(0.0) == 1.0
    assert oracle.exp_neg(-60.5) == 0.0
    assert oracle.exp_neg(-1e30) == 0.0


def test_exp_is_monotone_on_a_fine_grid(oracle):
    xs = np.linspace(-3.0, 0.0, 30001).astype(np.float32)
    ys = [oracle.exp_neg(float(x)) for x in xs]
    # a tiny slack for the polynomial's rounding, but no visible dips
    assert all(b >= a * (1 - 3e-7) for a, b in zip(ys, ys[1:]))


def test_weight_is_truncated_scaling(oracle):
    assert oracle.weight_of(1.0) == 1 << 40
    assert oracle.weight_of(0.0) == 0
    assert oracle.weight_of(2.0 ** -40) == 1
    assert oracle.weight_of(2.0 ** -41) == 0
    assert oracle.weight_of(1.5 * 2.0 ** -40) == 1


# ---------------------------------------------------------------- sampling row
def _double_reference(lc, lu, s, T, K):
    """CFG -> 1/T -> top-K (ties kept) -> softmax, in double precision with library routines."""
    z = (lu.astype(np.float64) + s * (lc.astype(np.float64) - lu.astype(np.float64))) / T
    if K < len(z):
        t = np.sort(z)[::-1][K - 1]
        keep = z >= t
    else:
        keep = np.ones(len(z), dtype=bool)
    zz = np.where(keep, z, -np.inf)
    p = np.exp(zz - zz.max())
    return p / p.sum(), keep


@pytest.mark.parametrize("V,K,s,T", [(64, 10, 3.0, 1.0), (1000, 100, 3.0, 1.0), (4096, 256, 3.0, 1.0),
                                      (513, 513, 1.5, 0.7), (300, 1000, 0.0, 2.0)])
def test_sampling_row_matches_double_softmax(oracle, V, K, s, T):
    rng = np.random.default_rng(V + K)
    lc = (rng.standard_normal(V) * 3).astype(np.float32)
    lu = (rng.standard_normal(V) * 3).astype(np.float32)
    e, Z = oracle.sampling_row(lc, lu, s, T, K)
    p_ref, keep = _double_reference(lc, lu, s, T, K)
    w = oracle.weights_of(e)
    assert int(w.sum()) == Z
    # same kept set (entries whose probability truncates to zero at 2^-40 aside); nothing outside it
    assert ((e > 0) == keep)[p_ref > 2.0 ** -36].all()
    assert not (e[~keep] > 0).any()
    p = w.astype(np.float64) / Z
    # fp32 guided logit (rel. 2^-23 of |z| ~ 30) + polynomial (4e-7) + truncation to 2^-40
    assert np.abs(p - p_ref).max() < 2e-5 * p_ref.max() + 2.0 ** -38
    assert abs(p.sum() - 1.0) < 1e-12


def test_top_k_equal_vocab_is_plain_softmax(oracle):
    rng = np.random.default_rng(5)
    l = rng.standard_normal(200).astype(np.float32)
    e, Z = oracle.sampling_row(l, l, 3.0, 1.0, 200)  # l_c == l_u: guidance is the identity
    p = oracle.weights_of(e).astype(np.float64) / Z
    ref = np.exp(l.astype(np.float64) - l.max())
    ref /= ref.sum()
    assert np.abs(p - ref).max() < 1e-6
    assert (e > 0).all()


def test_top_1_is_one_hot_at_argmax(oracle):
    rng = np.random.default_rng(6)
    lc = rng.standard_normal(333).astype(np.float32)
    lu = rng.standard_normal(333).astype(np.float32)
    e, Z = oracle.sampling_row(lc, lu, 3.0, 1.0, 1)
    z = lu.astype(np.float64) + 3.0 * (lc.astype(np.float64) - lu.astype(np.float64))
    assert (e > 0).sum() == 1 and int(np.argmax(e)) == int(np.argmax(z))
    assert Z == 1 << 40 and e.max() == 1.0


def test_top_k_keeps_ties_at_the_threshold(oracle):
    l = np.array([5, 4, 4, 4, 1, 0], dtype=np.float32)
    e, _ = oracle.sampling_row(l, l, 1.0, 1.0, 2)
    assert list(e > 0) == [True, True, True, True, False, False]


def test_guidance_formula_and_temperature(oracle):
    # two entries: z = l_u + s (l_c - l_u), scaled by 1/T; check the ratio of the two weights
    lc = np.array([1.0, 0.0], dtype=np.float32)
    lu = np.array([0.5, 1.0], dtype=np.float32)
    e, Z = oracle.sampling_row(lc, lu, 3.0, 2.0, 2)
    z = np.array([0.5 + 3 * 0.5, 1.0 + 3 * (-1.0)]) / 2.0
    assert abs(e[1] / e[0] - math.exp(z[1] - z[0])) < 1e-6


# ---------------------------------------------------------------- inverse CDF
def test_inverse_cdf_exhaustive_16_bit(oracle):
    # weights 2^40 * e with e dyadic, Z a power of two: every 16-bit uniform lands exactly in proportion
    e = np.array([0.5, 0.0, 0.25, 0.125, 0.0, 0.0625, 0.0625], dtype=np.float32)
    w = oracle.weights_of(e)
    Z = int(w.sum())
    assert Z == 1 << 40
    counts = np.zeros(len(e), dtype=np.int64)
    for u in range(1 << 16):
        counts[oracle.draw(e, Z, u << 48)] += 1
    assert list(counts) == [int(x) >> (40 - 16) for x in w]


def test_inverse_cdf_boundaries(oracle):
    e = np.array([0.25, 0.5, 0.25], dtype=np.float32)
    Z = 1 << 40
    assert oracle.draw(e, Z, 0) == 0
    assert oracle.draw(e, Z, (1 << 62) - 1) == 0      # just below 1/4
    assert oracle.draw(e, Z, 1 << 62) == 1            # exactly 1/4 goes to the next token
    assert oracle.draw(e, Z, (3 << 62) - 1) == 1
    assert oracle.draw(e, Z, 3 << 62) == 2
    assert oracle.draw(e, Z, (1 << 64) - 1) == 2


def test_residual_draw_exhaustive(oracle):
    # p = (1/2, 1/4, 1/4, 0), q = (1/4, 1/2, 0, 1/4): residual = (1/4, 0, 1/4, 0) -> tokens 0 and 2 equally
    ep = np.array([1.0, 0.5, 0.5, 0.0], dtype=np.float32)
    eq = np.array([0.5, 1.0, 0.0, 0.5], dtype=np.float32)
    Zp, Zq = int(oracle.weights_of(ep).sum()), int(oracle.weights_of(eq).sum())
    counts = np.zeros(4, dtype=np.int64)
    for u in range(1 << 12):
        counts[oracle.draw_residual(ep, Zp, eq, Zq, u << 52)] += 1
    assert list(counts) == [1 << 11, 0, 1 << 11, 0]
    # against the uniform reference (1/4 each): residual = (1/4, 0, 0, 0)
    assert {oracle.draw_residual(ep, Zp, None, 0, u << 52) for u in range(0, 1 << 12, 7)} == {0}
    # identical distributions: the residual is empty, the draw falls back to p
    got = [oracle.draw_residual(ep, Zp, ep, Zp, u << 52) for u in range(1 << 12)]
    assert got == [oracle.draw(ep, Zp, u << 52) for u in range(1 << 12)]


def test_residual_draw_against_a_one_hot_reference_exhaustive(oracle):
    """Eq. 3 with q = delta_x (a copied draft): max(0, p - q) is p with the entry of x removed (p(x) <= 1 = q(x)).
    p = (1/2, 1/4, 1/8, 1/8): without x = 0 the tokens 1, 2, 3 come in the ratio 2 : 1 : 1; without x = 2 the tokens
    0, 1, 3 in the ratio 4 : 2 : 1; exhaustively over 2^12 equally spaced uniforms (dyadic weights: exact counts)."""
    ep = np.array([1.0, 0.5, 0.25, 0.25], dtype=np.float32)
    Zp = int(oracle.weights_of(ep).sum())
    counts = np.zeros(4, dtype=np.int64)
    for u in range(1 << 12):
        counts[oracle.draw_residual_onehot(ep, Zp, 0, u << 52)] += 1
    assert list(counts) == [0, 1 << 11, 1 << 10, 1 << 10]
    counts[:] = 0
    for u in range(7 << 9):          # 7 * 512 cells of equal mass (residual mass 7/8 in units of 1/8), one uniform in the middle of each
        counts[oracle.draw_residual_onehot(ep, Zp, 2, ((2 * u + 1) << 64) // (7 << 10))] += 1
    assert list(counts) == [4 << 9, 2 << 9, 0, 1 << 9]
    # p itself one-hot at x: the residual is empty and the draw falls back to p
    one = np.array([0.0, 1.0, 0.0, 0.0], dtype=np.float32)
    Z1 = int(oracle.weights_of(one).sum())
    assert {oracle.draw_residual_onehot(one, Z1, 1, u << 52) for u in range(0, 1 << 12, 5)} == {1}
    # ... and it agrees with the general routine fed the one-hot row
    q = np.array([0.0, 0.0, 1.0, 0.0], dtype=np.float32)
    Zq = int(oracle.weights_of(q).sum())
    for u in range(0, 1 << 12, 3):
        assert oracle.draw_residual_onehot(ep, Zp, 2, u << 52) == oracle.draw_residual(ep, Zp, q, Zq, u << 52)


# ------------------------------------------------------- forced-token ranges
def test_a_token_range_is_the_plain_routine_on_the_sliced_row(oracle):
    """A forced-token mask gives ids outside [lo, hi) probability 0 before top-K: the masked row must equal the plain
    routine run on the slice, padded with zeros; the whole range is no mask; a range of one id is one-hot."""
    rng = np.random.default_rng(11)
    V, K = 300, 40
    lc = (rng.standard_normal(V) * 2).astype(np.float32)
    lu = (rng.standard_normal(V) * 2).astype(np.float32)
    full = oracle.sampling_row(lc, lu, 3.0, 0.9, K)
    same = oracle.sampling_row(lc, lu, 3.0, 0.9, K, allow=(0, V))
    assert np.array_equal(full[0], same[0]) and full[1] == same[1]
    for lo, hi in [(0, 50), (17, 200), (250, 300), (10, 30), (120, 121)]:
        e, Z = oracle.sampling_row(lc, lu, 3.0, 0.9, K, allow=(lo, hi))
        e_s, Z_s = oracle.sampling_row(lc[lo:hi], lu[lo:hi], 3.0, 0.9, K)
        assert Z == Z_s and np.array_equal(e[lo:hi], e_s)
        assert not e[:lo].any() and not e[hi:].any()
        assert (e > 0).sum() == min(K, hi - lo)
    e, Z = oracle.sampling_row(lc, lu, 3.0, 0.9, K, allow=(120, 121))
    assert e[120] == 1.0 and Z == 1 << 40


# ---------------------------------------------------------------- accept / keep
def test_accept_rule_against_exact_rationals(oracle):
    from fractions import Fraction
    rng = np.random.default_rng(9)
    for _ in range(2000):
        wp, wq = int(rng.integers(0, 1 << 40)), int(rng.integers(0, 1 << 40))
        Zp, Zq = int(rng.integers(1 << 40, 1 << 58)), int(rng.integers(1 << 40, 1 << 58))
        u = int(rng.integers(0, 1 << 32))
        r = Fraction(2 * u + 1, 1 << 33)
        exact = r * Fraction(wq, Zq) < Fraction(wp, Zp)
        margin = abs(float(r * Fraction(wq, Zq) - Fraction(wp, Zp)))
        if margin > 1e-12:  # away from a double-rounding tie the rule is Eq. 2 exactly
            assert oracle.accept(u, wp, Zp, wq, Zq) == exact
    assert oracle.accept(0xFFFFFFFF, 5, 10, 5, 10)        # p == q always accepts (r < 1)
    assert oracle.accept(0, 1 << 20, 1 << 50, 1 << 40, 1 << 41)      # r q = 2^-34 < p = 2^-30
    assert not oracle.accept(0, 1, 1 << 50, 1 << 40, 1 << 41)        # r q = 2^-34 > p = 2^-50
    assert not oracle.accept(123, 0, 10, 5, 10)           # p = 0 never accepts
    assert oracle.accept(123, 3, 10, 0, 10)               # q = 0 < p accepts
    assert not oracle.accept(123, 0, 10, 0, 10)           # 0 / 0 rejects


def test_keep_rule(oracle):
    assert oracle.keep(0.5, 6, 10, 10, 10)        # ratio 0.6 > 0.5
    assert not oracle.keep(0.5, 5, 10, 10, 10)    # ratio 0.5 is not > 0.5
    assert not oracle.keep(0.5, 4, 10, 10, 10)
    assert not oracle.keep(float("inf"), 10, 10, 1, 10)  # tau = +inf never keeps (no-reuse rule, Eq. 6)
    assert oracle.keep(0.0, 1, 10, 10, 10)        # tau = 0 keeps anything with p > 0
    assert not oracle.keep(0.0, 0, 10, 10, 10)


# ---------------------------------------------------------------- Theorem 1
def _row(oracle, logits, K):
    l = np.asarray(logits, dtype=np.float32)
    return oracle.sampling_row(l, l, 1.0, 1.0, K)


@pytest.mark.parametrize("V,seed", [(2, 0), (3, 1), (5, 2), (8, 3), (8, 4)])
def test_theorem1_accept_plus_residual_reproduces_p(oracle, V, seed):
    """x ~ q, accept w.p. min(1, p/q), else residual draw: the result is distributed as p (appendix, Theorem 1);
    the rejection probability is sum max(0, p - q)."""
    rng = np.random.default_rng(seed)
    ep, Zp = _row(oracle, rng.standard_normal(V) * 1.5, max(1, V - seed % 2))
    eq, Zq = _row(oracle, rng.standard_normal(V) * 1.5, V)
    p = oracle.weights_of(ep).astype(np.float64) / Zp
    q = oracle.weights_of(eq).astype(np.float64) / Zq
    n = 1_000_000
    counts, rejected = oracle.law_trials(ep, Zp, eq, Zq, seed + 77, n)
    assert counts.sum() == n
    support = p > 0
    assert counts[~support].sum() == 0
    chi = stats.chisquare(counts[support], p[support] * n)
    assert chi.pvalue > 0.01, (counts, p * n)
    # brute-force law of the two-branch procedure equals p term by term (the identity used in the proof)
    law = np.minimum(p, q) + (1 - np.minimum(p, q).sum()) * np.maximum(0, p - q) / max(np.maximum(0, p - q).sum(), 1e-300)
    assert np.abs(law - p).max() < 1e-12
    rate = np.maximum(0, p - q).sum()
    sigma = math.sqrt(max(rate * (1 - rate), 1e-12) / n)
    assert abs(rejected / n - rate) < 5 * sigma + 1e-6


def test_theorem1_with_uniform_reference(oracle):
    V = 7
    ep, Zp = _row(oracle, [2.0, 0.1, -1.0, 0.5, 0.0, 1.0, -3.0], 5)
    p = oracle.weights_of(ep).astype(np.float64) / Zp
    n = 1_000_000
    counts, rejected = oracle.law_trials(ep, Zp, None, 0, 5, n)
    support = p > 0
    assert counts[~support].sum() == 0
    assert stats.chisquare(counts[support], p[support] * n).pvalue > 0.01
    rate = np.maximum(0, p - 1.0 / V).sum()
    assert abs(rejected / n - rate) < 5 * math.sqrt(rate * (1 - rate) / n)


def test_equal_distributions_never_reject(oracle):
    ep, Zp = _row(oracle, [0.3, -0.2, 1.1, 0.0, 2.0], 5)
    counts, rejected = oracle.law_trials(ep, Zp, ep, Zp, 1, 200_000)
    assert rejected == 0


def test_a_mistaken_residual_would_be_caught(oracle):
    """Sensitivity check of the chi-square pin: drawing the rejected token from p instead of the residual
    (a plausible mistake) gives a law the same test rejects decisively."""
    rng = np.random.default_rng(2)
    V = 5
    ep, Zp = _row(oracle, rng.standard_normal(V) * 1.5, V)
    eq, Zq = _row(oracle, rng.standard_normal(V) * 1.5, V)
    p = oracle.weights_of(ep).astype(np.float64) / Zp
    q = oracle.weights_of(eq).astype(np.float64) / Zq
    wrong = np.minimum(p, q) + (1 - np.minimum(p, q).sum()) * p
    n = 1_000_000
    expected_stat = n * ((wrong - p) ** 2 / p).sum()
    assert expected_stat > 200  # far beyond the p = 0.01 critical value (~13 for 4 dof)
