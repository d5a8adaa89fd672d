"""Pins for the oracle's single-token resample against what the paper and the
mathematics fix: the closed-form conditional (Eq. 1), the split p = p1 + p2
with S and Q (Eq. 6-7), the one-uniform bucket rule and the "smallest k whose
prefix sum exceeds the draw" search (Section 6.1.1), and special cases that
reduce to textbook urns."""
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

import oracle


def make_state(rng, K, V, n_doc, n_word, n_other, o=None):
    """A consistent frozen state around one token: its document has n_doc
    tokens, its word n_word tokens, and n_other further tokens exist elsewhere.
    Returns dense rows n_d, n_w, n_k (all including the token) and its topic."""
    o = int(rng.integers(K)) if o is None else o
    n_d = np.bincount(rng.integers(K, size=n_doc - 1), minlength=K).astype(np.int32)
    n_w = np.bincount(rng.integers(K, size=n_word - 1), minlength=K).astype(np.int32)
    n_d[o] += 1
    n_w[o] += 1
    n_k = n_w + np.bincount(rng.integers(K, size=n_other), minlength=K).astype(np.int32)
    return n_d, n_w, n_k, o


def closed_form(K, V, alpha, beta, n_d, n_w, n_k, o):
    """Eq. 1 with the token itself removed, normalised (fp64)."""
    e = np.zeros(K); e[o] = 1
    p = (n_d - e + alpha) * (n_w - e + beta) / (n_k - e + beta * V)
    return p / p.sum()


def draw_many(K, V, alpha, beta, n_d, n_w, n_k, o, n, seed=11):
    u = oracle.uniforms(seed, 1, 0, n)
    return np.array([oracle.resample_token(K, V, alpha, beta, n_d, n_w, n_k, o, ui)[0]
                     for ui in u])


CASES = [
    # K, V, n_doc, n_word, n_other, alpha, beta
    (4, 5, 6, 3, 10, 0.5, 0.01),
    (8, 6, 12, 4, 30, 50 / 8, 0.01),
    (16, 50, 40, 25, 300, 50 / 16, 0.01),
    (32, 20, 5, 2, 40, 0.1, 0.5),
]


@pytest.mark.parametrize("case", CASES)
def test_draw_frequencies_follow_eq1(case):
    K, V, n_doc, n_word, n_other, alpha, beta = case
    rng = np.random.default_rng(sum(case[:5]))
    n_d, n_w, n_k, o = make_state(rng, K, V, n_doc, n_word, n_other)
    p = closed_form(K, V, alpha, beta, n_d, n_w, n_k, o)
    z = draw_many(K, V, alpha, beta, n_d, n_w, n_k, o, 120_000)
    obs = np.bincount(z, minlength=K)
    keep = p * len(z) >= 5
    f_obs = np.append(obs[keep], obs[~keep].sum())
    f_exp = np.append(p[keep], p[~keep].sum()) * len(z)
    if f_exp[-1] == 0:
        f_obs, f_exp = f_obs[:-1], f_exp[:-1]
    assert stats.chisquare(f_obs, f_exp).pvalue > 1e-4


def test_own_count_is_excluded_where_it_matters_most():
    # The token is the only one of its topic anywhere: after exclusion theta, phi and
    # n_k are all 0 there, so p(o) = alpha*beta/(beta V) = alpha/V, far below what the
    # unexcluded counts would give.
    K, V, alpha, beta = 3, 4, 0.2, 0.01
    n_d = np.array([1, 5, 0], np.int32); n_w = np.array([1, 0, 2], np.int32)
    n_k = np.array([1, 9, 7], np.int32); o = 0
    p = closed_form(K, V, alpha, beta, n_d, n_w, n_k, o)
    assert abs(p[0] * ((5.2 * 0.01 / 9.04) + (0.2 * 2.01 / 7.04) + 0.05) - 0.05) < 1e-12
    z = draw_many(K, V, alpha, beta, n_d, n_w, n_k, o, 60_000)
    obs = np.bincount(z, minlength=K)
    assert stats.chisquare(obs, p * len(z)).pvalue > 1e-4
    wrong = (n_d + alpha) * (n_w + beta) / (n_k + beta * V)          # no exclusion
    assert stats.chisquare(obs, wrong / wrong.sum() * len(z)).pvalue < 1e-12


@pytest.mark.parametrize("case", CASES)
def test_S_plus_Q_is_the_dense_normaliser(case):
    K, V, n_doc, n_word, n_other, alpha, beta = case
    rng = np.random.default_rng(1 + sum(case[:5]))
    n_d, n_w, n_k, o = make_state(rng, K, V, n_doc, n_word, n_other)
    _, S, Q = oracle.resample_token(K, V, alpha, beta, n_d, n_w, n_k, o, 0.5)
    e = np.zeros(K); e[o] = 1
    pstar = ((n_w - e + beta) / (n_k - e + beta * V)).astype(np.float32).astype(np.float64)
    dense = ((n_d - e + alpha) * pstar).sum()
    assert abs((S + Q) - dense) <= 1e-12 * dense
    assert abs(S - ((n_d - e) * pstar).sum()) <= 1e-12 * max(S, 1e-300)
    # bucket frequency ~ S/(S+Q)
    u = oracle.uniforms(5, 1, 0, 20000)
    in_sparse = (u * (S + Q) < S).mean()
    assert abs(in_sparse - S / (S + Q)) < 4 * np.sqrt(0.25 / len(u))


def exact_intervals(K, V, alpha, beta, n_d, n_w, n_k, o):
    """The concatenated CDF [p1 ascending k | p2 ascending k] in exact rational
    arithmetic, from the canonical fp32 weights.  Returns (topic, lo, hi) with
    lo, hi in u-space, zero-width intervals dropped."""
    e = np.zeros(K); e[o] = 1
    pstar = ((n_w - e + beta) / (n_k - e + beta * V)).astype(np.float32)
    w = [Fraction(float(x)) for x in pstar]
    parts = [(k, int(n_d[k] - e[k]) * w[k]) for k in range(K)]
    parts += [(k, Fraction(alpha) * w[k]) for k in range(K)]
    total = sum(x for _, x in parts)
    out, acc = [], Fraction(0)
    for k, x in parts:
        if x > 0:
            out.append((k, acc / total, (acc + x) / total))
        acc += x
    return out


@pytest.mark.parametrize("case", CASES)
def test_inverse_cdf_matches_exact_rational_boundaries(case):
    K, V, n_doc, n_word, n_other, alpha, beta = case
    rng = np.random.default_rng(2 + sum(case[:5]))
    n_d, n_w, n_k, o = make_state(rng, K, V, n_doc, n_word, n_other)
    checked = 0
    for k, lo, hi in exact_intervals(K, V, alpha, beta, n_d, n_w, n_k, o):
        width = float(hi - lo)
        if width < 1e-9:
            continue
        for frac in (Fraction(1, 1000), Fraction(1, 2), Fraction(999, 1000)):
            u = float(lo + (hi - lo) * frac)
            got, _, _ = oracle.resample_token(K, V, alpha, beta, n_d, n_w, n_k, o, u)
            assert got == k, (k, got, u)
            checked += 1
    assert checked >= 3 * K          # the dense bucket alone has K intervals
    assert oracle.resample_token(K, V, alpha, beta, n_d, n_w, n_k, o, 0.0)[0] == \
        exact_intervals(K, V, alpha, beta, n_d, n_w, n_k, o)[0][0]
    assert oracle.resample_token(K, V, alpha, beta, n_d, n_w, n_k, o, 1 - 2.0**-53)[0] == K - 1


def test_single_topic_always_zero():
    n = np.array([7], np.int32)
    for u in (0.0, 0.3, 0.999999):
        assert oracle.resample_token(1, 9, 50.0, 0.01, n, n, n + 5, 0, u)[0] == 0


def test_single_token_document_takes_dense_bucket():
    # theta' is all zero: S = 0, every draw comes from p2 ~ p*
    K, V, alpha, beta = 5, 7, 0.3, 0.01
    n_d = np.array([0, 0, 1, 0, 0], np.int32)
    n_w = np.array([3, 0, 1, 8, 1], np.int32); n_k = n_w + np.array([4, 2, 0, 9, 1], np.int32)
    k, S, Q = oracle.resample_token(K, V, alpha, beta, n_d, n_w, n_k, 2, 0.0)
    assert S == 0.0 and k == 0
    p = closed_form(K, V, alpha, beta, n_d, n_w, n_k, 2)
    z = draw_many(K, V, alpha, beta, n_d, n_w, n_k, 2, 40_000)
    assert stats.chisquare(np.bincount(z, minlength=K), p * len(z)).pvalue > 1e-4


@pytest.mark.parametrize("V,beta", [(1, 0.01), (9, 1e12)])
def test_reduces_to_document_urn(V, beta):
    """With one word in the vocabulary (phi_k = n_k, so p* = 1), or with beta so large
    that p* rounds to the same fp32 for every topic, Eq. 1 is the Polya urn of the
    document alone: p(k) ~ theta'_dk + alpha.  The draw is then known exactly: position
    x = u (N_d - 1 + K alpha) either indexes the document's other tokens sorted by topic,
    or, past them, a uniform topic."""
    K, alpha = 6, 0.75
    rng = np.random.default_rng(V)
    z_doc = rng.integers(K, size=15)
    n_d = np.bincount(z_doc, minlength=K).astype(np.int32)
    o = int(z_doc[0])
    if V == 1:
        n_w = n_d + 3
        n_k = n_w.copy()
    else:
        n_w = np.bincount(rng.integers(K, size=8), minlength=K).astype(np.int32); n_w[o] += 1
        n_k = n_w + 5
    others = np.sort(z_doc[1:])
    n_others = len(others)
    for u in np.linspace(0.003, 0.997, 211):
        x = u * (n_others + K * alpha)
        frac = x - np.floor(x) if x < n_others else ((x - n_others) / alpha) % 1.0
        if min(frac, 1 - frac) < 1e-6:
            continue
        want = others[int(x)] if x < n_others else int((x - n_others) / alpha)
        got, S, Q = oracle.resample_token(K, V, alpha, beta, n_d, n_w, n_k, o, float(u))
        assert got == want
        # S/Q = (N_d - 1)/(K alpha): the common factor p* cancels
        assert abs(S / Q - n_others / (K * alpha)) < 1e-9


def test_large_alpha_reduces_to_word_side():
    # alpha -> infinity: p(k) -> p*'(k) = (phi'_kv + beta)/(n'_k + beta V), normalised
    K, V, alpha, beta = 6, 11, 1e12, 0.01
    rng = np.random.default_rng(3)
    n_d, n_w, n_k, o = make_state(rng, K, V, 9, 14, 60)
    e = np.zeros(K); e[o] = 1
    p = (n_w - e + beta) / (n_k - e + beta * V)
    z = draw_many(K, V, alpha, beta, n_d, n_w, n_k, o, 60_000)
    assert stats.chisquare(np.bincount(z, minlength=K), p / p.sum() * len(z)).pvalue > 1e-4
