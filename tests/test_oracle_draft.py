"""Pins for the oracle's draft-side candidate sampler (Sec. 3.1; Eq. (1) for sampling
without replacement).  None of these re-types the oracle's own routine: they use the measure
of the uniforms that map to each outcome, numpy's cumulative-sum search, and the law of the
whole method (candidates from the sampler, then Algorithm 1 / 2, give the target distribution)."""
import itertools

import numpy as np
import pytest

from oracle import mcsd_oracle as O

WITH, WITHOUT = 0, 1


def _rand_dist(rng, V, conc=1.0):
    return rng.dirichlet(np.full(V, conc))


def _logits(p):
    return np.log(p).astype(np.float32)


def _softmax64(z, T=1.0):
    z = z.astype(np.float64) / T
    e = np.exp(z - z.max())
    return e / e.sum()


def test_single_draw_measure_equals_q():
    # the set of uniforms mapped to token x has measure q(x): midpoints of a fine grid
    rng = np.random.default_rng(11)
    V, G = 7, 40000
    z = _logits(_rand_dist(rng, V))
    q = _softmax64(z)
    u = (np.arange(G) + 0.5) / G
    counts = np.zeros(V)
    for ui in u:
        tok, _ = O.draft_parent(z, [ui], 1, WITH)
        counts[tok[0]] += 1
    # every CDF boundary can misplace at most one grid cell (float32 uniforms: a second one)
    assert np.abs(counts / G - q).max() <= 3.0 / G + 1e-6


@pytest.mark.parametrize("variant", [WITH, WITHOUT])
def test_pair_measure_matches_product_or_eq1(variant):
    # k = 2: measure of (u1, u2) mapped to (x1, x2) is q(x1) q(x2) with replacement and
    # q(x1) q(x2) / (1 - q(x1)) for x2 != x1 without (Eq. (1)), zero on the diagonal
    rng = np.random.default_rng(12 + variant)
    V, G = 4, 500
    z = _logits(_rand_dist(rng, V))
    q = _softmax64(z)
    freq = np.zeros((V, V))
    grid = (np.arange(G) + 0.5) / G
    for u1 in grid:
        for u2 in grid:
            tok, _ = O.draft_parent(z, [u1, u2], 2, variant)
            freq[tok[0], tok[1]] += 1
    freq /= G * G
    want = np.outer(q, q)
    if variant == WITHOUT:
        want = np.outer(q / (1.0 - q), q)
        np.fill_diagonal(want, 0.0)
        assert np.all(np.diag(freq) == 0.0)
    assert np.abs(freq - want).max() <= 4.0 / G


def test_triple_without_replacement_matches_eq1_chain():
    # third draw: q(x3) / (1 - q(x1) - q(x2)), conditional on the first two (Eq. (1))
    rng = np.random.default_rng(14)
    V, G = 4, 2000
    z = _logits(_rand_dist(rng, V))
    q = _softmax64(z)
    grid = (np.arange(G) + 0.5) / G
    # fix u1, u2 so that (x1, x2) = (2, 0); sweep u3
    cdf = np.cumsum(q)
    u1 = (cdf[1] + cdf[2]) / 2
    qbar1 = q.copy(); qbar1[2] = 0; qbar1 /= qbar1.sum()
    u2 = qbar1[0] / 2
    counts = np.zeros(V)
    for u3 in grid:
        tok, _ = O.draft_parent(z, [u1, u2, u3], 3, WITHOUT)
        assert tok[0] == 2 and tok[1] == 0
        counts[tok[2]] += 1
    want = q.copy(); want[[2, 0]] = 0; want /= (1.0 - q[2] - q[0])
    assert np.abs(counts / G - want).max() <= 3.0 / G


@pytest.mark.parametrize("variant", [WITH, WITHOUT])
@pytest.mark.parametrize("T", [1.0, 0.7, 2.5])
def test_against_numpy_cumsum_search(variant, T):
    rng = np.random.default_rng(15)
    V, k = 3000, 6
    for trial in range(20):
        z = (3.0 * rng.standard_normal(V)).astype(np.float32)
        u = rng.random(k).astype(np.float32)
        tok, margin = O.draft_parent(z, u, k, variant, T=T)
        q = _softmax64(z, T)
        for i in range(k):
            cdf = np.cumsum(q)
            x = int(np.searchsorted(cdf, float(u[i]), side="right"))
            if margin[i] > 1e-9:      # away from a CDF edge the two summation orders agree
                assert tok[i] == x, (trial, i)
            if variant == WITHOUT:
                q[tok[i]] = 0.0
                q /= q.sum()
        if variant == WITHOUT:
            assert len(set(tok.tolist())) == k


def test_temperature_zero_is_top_k_lowest_id_first():
    rng = np.random.default_rng(16)
    V, k = 500, 8
    z = rng.integers(-5, 5, V).astype(np.float32)        # many ties
    tok, margin = O.draft_parent(z, np.zeros(k, np.float32), k, WITHOUT, T=0.0)
    order = np.lexsort((np.arange(V), -z.astype(np.float64)))
    np.testing.assert_array_equal(tok, order[:k])
    assert np.all(np.isinf(margin))


def test_same_uniform_with_replacement_repeats_token():
    z = _logits(np.array([0.1, 0.2, 0.3, 0.4]))
    tok, _ = O.draft_parent(z, [0.55, 0.55, 0.55], 3, WITH)
    assert tok.tolist() == [2, 2, 2]
    tok, _ = O.draft_parent(z, [0.55, 0.55, 0.55], 3, WITHOUT)
    assert len(set(tok.tolist())) == 3


@pytest.mark.parametrize("variant", [WITH, WITHOUT])
def test_sampler_then_verification_returns_target_distribution(variant):
    # Theorem of Appendix A / B end to end by Monte Carlo: candidates from the sampler, one
    # round of Algorithm 1 / 2, the emitted token (accepted candidate or endpoint) follows p.
    rng = np.random.default_rng(17 + variant)
    V, k, n = 4, 3, 60000
    p = _rand_dist(rng, V)
    q = _rand_dist(rng, V)
    zp, zq = _logits(p), _logits(q)
    p64 = _softmax64(zp)
    counts = np.zeros(V)
    for _ in range(n):
        u = rng.random(2 * k + 1).astype(np.float32)
        tok, _ = O.draft_parent(zq, u[:k], k, variant)
        res = O.verify_parent(zp, zq, tok, u[k:2 * k], float(u[2 * k]), variant, T=1.0)
        counts[tok[res.accepted] if res.accepted >= 0 else res.endpoint] += 1
    sigma = np.sqrt(p64 * (1 - p64) / n)
    assert np.all(np.abs(counts / n - p64) <= 4.5 * sigma + 1e-4)


def test_tree_level_sampler_places_draws_on_children():
    rng = np.random.default_rng(19)
    parent = np.array([-1, -1, 0, 0, 0, 1, 3], np.int32)      # root: 0,1; node 0: 2,3,4; node 1: 5; node 3: 6
    N, V, B = 7, 50, 3
    q_row = np.array([0, 1, 2, -1, 3, -1, -1, -1], np.int32)   # rows with children: 0, 1, 2, 4
    P = 4
    draft = (2.0 * rng.standard_normal((B, P, V))).astype(np.float32)
    u = rng.random((B, N)).astype(np.float32)
    temp = np.array([1.0, 0.0, 0.5], np.float32)
    cand, margin = O.draft_sample(draft, q_row, parent, u, temp, WITHOUT, n_threads=2)
    kids = {0: [0, 1], 1: [2, 3, 4], 2: [5], 4: [6]}
    for b in range(B):
        for row, ch in kids.items():
            tok, mg = O.draft_parent(draft[b, q_row[row]], u[b, ch], len(ch), WITHOUT, T=float(temp[b]))
            np.testing.assert_array_equal(cand[b, ch], tok)
            np.testing.assert_array_equal(margin[b, ch], mg)


def test_bad_draft_row_map_is_an_error():
    parent = np.array([-1, 0], np.int32)
    q_row = np.array([0, 5, -1], np.int32)       # row 1 has a child but its draft row is out of range
    with pytest.raises(ValueError):
        O.draft_sample(np.zeros((1, 2, 8), np.float32), q_row, parent, np.full((1, 2), 0.5, np.float32),
                       np.ones(1, np.float32), WITH)
