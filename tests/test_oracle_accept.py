"""Pins for the speculative-acceptance oracle.

What fixes it from outside: the greedy special case (longest matching prefix), losslessness
(the emitted token follows the target distribution -- Monte Carlo), the closed-form acceptance
probability sum(min(p, q)), an independent exact-integer sampler written with Python ints,
and an exhaustive sweep over all 2^24 uniforms of one row.
"""
from fractions import Fraction
from itertools import product

import numpy as np
import pytest

import synth_inputs as S


def rand_dist(g, *shape):
    x = g.random(shape) ** 3 + 1e-3
    return (x / x.sum(-1, keepdims=True)).astype(np.float32)


def py_weight(r32) -> int:
    """trunc(r * 2^40) in exact rational arithmetic."""
    return int(Fraction(float(np.float32(r32))) * (1 << 40))


def py_sample(row_p, row_q, u) -> int:
    """Inverse CDF on the integer weights, in Python integers only."""
    if row_q is None:
        r = [np.float32(x) for x in row_p]
    else:
        r = [max(np.float32(0), np.float32(a) - np.float32(b)) for a, b in zip(row_p, row_q)]
    w = [py_weight(x) for x in r]
    Z = sum(w)
    if Z == 0:
        return -1
    m = int(Fraction(float(np.float32(u))) * (1 << 24))
    T = (m * Z) >> 24
    run = 0
    for v, wv in enumerate(w):
        run += wv
        if run > T:
            return v
    raise AssertionError("T < Z must hold")


# ---------------------------------------------------------------- greedy special case
def test_greedy_accepts_exactly_the_longest_matching_prefix(oracle):
    V, k = 3, 2
    eye = np.eye(V, dtype=np.float32)
    us = [0.0, 0.25, 0.999999]
    cases = []
    for tp in product(range(V), repeat=k + 1):          # argmax of p_0..p_k
        for x in product(range(V), repeat=k):           # draft tokens = argmax of q_j (greedy draft)
            for u in product(us, repeat=k + 1):
                cases.append((tp, x, u))
    p = np.stack([eye[list(tp)] for tp, _, _ in cases])
    q = np.stack([eye[list(x)] for _, x, _ in cases])
    d = np.array([x for _, x, _ in cases], np.int32)
    u = np.array([uu for _, _, uu in cases], np.float32)
    n, t = oracle.spec_accept(p, q, d, u)
    for c, (tp, x, _) in enumerate(cases):
        want = 0
        while want < k and tp[want] == x[want]:
            want += 1
        assert n[c] == want
        assert t[c] == tp[want]                          # correction (or bonus) = the target's argmax


# ---------------------------------------------------------------- losslessness, Monte Carlo
@pytest.mark.parametrize("k", [1, 2, 3])
def test_lossless_monte_carlo(oracle, k):
    """The token emitted at position j (draft j if accepted, else the resample, else the bonus)
    is distributed as the target p_j, whatever q is."""
    V, N = 8, 600_000
    g = np.random.default_rng(100 + k)
    p1 = rand_dist(g, k + 1, V)
    q1 = rand_dist(g, k, V)
    draft = np.stack([g.choice(V, size=N, p=q1[j].astype(np.float64) / q1[j].astype(np.float64).sum())
                      for j in range(k)], 1).astype(np.int32)
    u = (g.integers(0, 1 << 24, size=(N, k + 1)) / float(1 << 24)).astype(np.float32)
    p = np.ascontiguousarray(np.broadcast_to(p1, (N, k + 1, V)))
    q = np.ascontiguousarray(np.broadcast_to(q1, (N, k, V)))
    n, t = oracle.spec_accept(p, q, draft, u)
    assert n.min() >= 0 and n.max() <= k and t.min() >= 0 and t.max() < V
    # closed form: P[accept draft 0] = sum_v min(p_0(v), q_0(v))
    alpha = [float(np.minimum(p1[j], q1[j]).astype(np.float64).sum()) for j in range(k)]
    sig = np.sqrt(alpha[0] * (1 - alpha[0]) / N)
    assert abs((n >= 1).mean() - alpha[0]) < 4.5 * sig
    # E[accepted] = sum_j prod_{i<=j} alpha_i
    want_mean = sum(np.prod(alpha[:j + 1]) for j in range(k))
    assert abs(n.mean() - want_mean) < 4.5 * k / np.sqrt(N)
    for j in range(k + 1):
        reached = n >= j
        emitted = np.where(n > j, draft[:, min(j, k - 1)], t)[reached]
        cnt = np.bincount(emitted, minlength=V).astype(np.float64)
        M = cnt.sum()
        pj = p1[j].astype(np.float64) / p1[j].astype(np.float64).sum()
        chi2 = ((cnt - M * pj) ** 2 / (M * pj)).sum()
        assert chi2 < 35.0, (j, chi2)                    # 7 dof: P[chi2 > 35] ~ 1e-5
        assert np.abs(cnt / M - pj).max() < 5 * np.sqrt(0.25 / M)


def test_identical_distributions_accept_everything(oracle):
    V, k, N = 16, 4, 2000
    g = np.random.default_rng(7)
    p = rand_dist(g, N, k + 1, V)
    q = p[:, :k].copy()
    draft = g.integers(0, V, size=(N, k)).astype(np.int32)
    u = g.random((N, k + 1)).astype(np.float32)
    u[:, :k] = np.minimum(u[:, :k], np.float32(0.9999999))
    n, t = oracle.spec_accept(p, q, draft, u)
    assert (n == k).all()
    for b in range(0, N, 97):
        assert t[b] == py_sample(p[b, k], None, u[b, k])


# ---------------------------------------------------------------- the integer sampler
def test_k0_is_plain_inverse_cdf(oracle):
    V, N = 37, 3000
    g = np.random.default_rng(11)
    p = rand_dist(g, N, 1, V)
    u = (g.integers(0, 1 << 24, size=(N, 1)) / float(1 << 24)).astype(np.float32)
    n, t = oracle.spec_accept(p, None, None, u)
    assert (n == 0).all()
    w = np.floor(p[:, 0].astype(np.float64) * float(1 << 40)).astype(np.int64)      # exact: fp32 * 2^40 fits fp64
    for b in range(N):
        c = np.cumsum(w[b])
        m = int(u[b, 0] * (1 << 24))
        T = (m * int(c[-1])) >> 24
        assert t[b] == int(np.searchsorted(c, T, side="right"))


def test_resample_matches_python_integer_sampler(oracle):
    V, k, N = 11, 3, 4000
    g = np.random.default_rng(13)
    p = rand_dist(g, N, k + 1, V)
    q = rand_dist(g, N, k, V)
    # sprinkle exact zeros and tiny values, which must never be chosen / must round to weight 0
    p[:, :, 3] = 0.0
    q[:, :, 5] = 0.0
    p[:, :, 7] = np.float32(2.0 ** -41)
    draft = g.integers(0, V, size=(N, k)).astype(np.int32)
    u = (g.integers(0, 1 << 24, size=(N, k + 1)) / float(1 << 24)).astype(np.float32)
    n, t = oracle.spec_accept(p, q, draft, u)
    for b in range(N):
        want_n = 0
        while want_n < k and (Fraction(float(u[b, want_n])) * Fraction(float(q[b, want_n, draft[b, want_n]]))
                              < Fraction(float(p[b, want_n, draft[b, want_n]]))):
            want_n += 1
        assert n[b] == want_n
        want_t = py_sample(p[b, want_n], q[b, want_n] if want_n < k else None, u[b, k])
        assert t[b] == want_t
        if want_n < k:
            assert p[b, want_n, t[b]] > q[b, want_n, t[b]]     # only tokens with residual mass


def test_weight_rounding_edges(oracle):
    """w = trunc(r * 2^40): 2^-40 -> 1, just below -> 0, 1.0 -> 2^40; checked through which
    uniforms select which of two tokens."""
    tiny, below = np.float32(2.0 ** -40), np.float32(np.nextafter(np.float32(2.0 ** -40), np.float32(0)))
    # token 0 weight 1, token 1 weight 2^40: only m = 0 gives T = 0 < 1 -> token 0
    p = np.array([[[tiny, 1.0]]], np.float32)
    for m, want in ((0, 0), (1, 1), (12345, 1), ((1 << 24) - 1, 1)):
        _, t = oracle.spec_accept(p, None, None, np.array([[m / float(1 << 24)]], np.float32))
        assert t[0] == want
    # weight 0: token 0 can never be drawn, not even by u = 0
    p = np.array([[[below, 1.0]]], np.float32)
    _, t = oracle.spec_accept(p, None, None, np.array([[0.0]], np.float32))
    assert t[0] == 1
    # denormal residuals count as zero
    p = np.array([[[1e-40, 0.5, 1e-39]]], np.float32)
    for uu in (0.0, 0.5, 0.9999999):
        _, t = oracle.spec_accept(p, None, None, np.array([[uu]], np.float32))
        assert t[0] == 1


def test_exhaustive_uniforms_one_row(oracle):
    """All 2^24 values of m on one residual row: the number that pick token v is 2^24 * w_v / Z
    up to +-1, and exactly 0 where w_v = 0; the pick is monotone in m."""
    V, k = 6, 1
    p1 = np.array([[0.30, 0.05, 0.25, 0.0, 0.15, 0.25], [1 / 6] * 6], np.float32)
    q1 = np.array([[0.10, 0.25, 0.05, 0.3, 0.15, 0.15]], np.float32)
    x = 3                                               # p(x) = 0: rejected for every u
    w = [py_weight(max(np.float32(0), p1[0, v] - q1[0, v])) for v in range(V)]
    Z = sum(w)
    counts = np.zeros(V, np.int64)
    chunk = 1 << 20
    last = 0
    for c in range(16):
        m = np.arange(c * chunk, (c + 1) * chunk, dtype=np.int64)
        u = np.empty((chunk, 2), np.float32)
        u[:, 0] = 0.0
        u[:, 1] = (m / float(1 << 24)).astype(np.float32)
        p = np.ascontiguousarray(np.broadcast_to(p1, (chunk, 2, V)))
        q = np.ascontiguousarray(np.broadcast_to(q1, (chunk, 1, V)))
        n, t = oracle.spec_accept(p, q, np.full((chunk, 1), x, np.int32), u)
        assert (n == 0).all()
        assert (np.diff(t) >= 0).all() and t[0] >= last
        last = t[-1]
        counts += np.bincount(t, minlength=V)
    assert counts.sum() == 1 << 24
    for v in range(V):
        if w[v] == 0:
            assert counts[v] == 0
        else:
            assert abs(counts[v] - Fraction((1 << 24) * w[v], Z)) <= 1
    assert counts[1] == 0 and counts[3] == 0 and counts[4] == 0      # p <= q there


def test_u_extremes(oracle):
    p = np.array([[[0.0, 0.2, 0.0, 0.5, 0.3, 0.0]]], np.float32)
    _, t = oracle.spec_accept(p, None, None, np.array([[0.0]], np.float32))
    assert t[0] == 1                                    # first token with mass
    _, t = oracle.spec_accept(p, None, None, np.array([[np.nextafter(np.float32(1), np.float32(0))]], np.float32))
    assert t[0] == 4                                    # last token with mass


def test_accept_boundary_is_strict(oracle):
    """u*q < p, strictly: u = p/q exactly is a rejection, u = 0 with p(x) = 0 is a rejection,
    q(x) = 0 < p(x) is an acceptance."""
    p = np.array([[[0.25, 0.75], [0.5, 0.5]]], np.float32)
    q = np.array([[[0.5, 0.5]]], np.float32)
    d = np.array([[0]], np.int32)
    n, _ = oracle.spec_accept(p, q, d, np.array([[0.5, 0.1]], np.float32))
    assert n[0] == 0
    n, _ = oracle.spec_accept(p, q, d, np.array([[np.nextafter(np.float32(0.5), np.float32(0)), 0.1]], np.float32))
    assert n[0] == 1
    p0 = np.array([[[0.0, 1.0], [0.5, 0.5]]], np.float32)
    n, t = oracle.spec_accept(p0, q, d, np.array([[0.0, 0.1]], np.float32))
    assert n[0] == 0 and t[0] == 1
    q0 = np.array([[[0.0, 1.0]]], np.float32)
    n, _ = oracle.spec_accept(p, q0, d, np.array([[0.99, 0.1]], np.float32))
    assert n[0] == 1


def test_degenerate_rows(oracle):
    # rejected although p == q (p(x) = q(x) = 0): the residual is empty, the row p is sampled
    p = np.array([[[0.0, 0.5, 0.5], [1.0, 0.0, 0.0]]], np.float32)
    q = p[:, :1].copy()
    n, t = oracle.spec_accept(p, q, np.array([[0]], np.int32), np.array([[0.3, 0.75]], np.float32))
    assert n[0] == 0 and t[0] == py_sample(p[0, 0], None, 0.75) == 2
    # nothing to sample at all
    z = np.zeros((1, 2, 3), np.float32)
    n, t = oracle.spec_accept(z, z[:, :1], np.array([[0]], np.int32), np.array([[0.3, 0.75]], np.float32))
    assert n[0] == 0 and t[0] == -1


def test_synthetic_draft_hits_the_papers_acceptance_band(oracle):
    """The correlated-logit draft of the workload recipe accepts at 2*Phi(-sigma/2): 0.80 for
    sigma = 0.5, inside the 0.70 - 0.90 the paper measures for its model pairs (Appendix)."""
    cfg = S.CONFIGS["C2"].with_(B=8, V=20000)
    s = S.accept_inputs(cfg)
    alpha = np.minimum(s["p"][:, :cfg.k], s["q"]).astype(np.float64).sum(-1).mean()
    assert abs(alpha - S.expected_acceptance(0.5)) < 0.02
    assert 0.70 < alpha < 0.90
    n, t = oracle.spec_accept(s["p"], s["q"], s["draft"], s["u"])
    assert ((0 <= n) & (n <= cfg.k)).all() and ((0 <= t) & (t < cfg.V)).all()
