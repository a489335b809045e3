"""Pins for the logits-input acceptance oracle (softmax defined on integers).

Outside references: 2**t / scipy softmax for the integer weights, the probability-input
oracle (itself pinned) for the decisions, the greedy limit, Monte-Carlo losslessness, an exact
power-of-two invariance, and a Python big-integer re-computation of the decision logic from the
oracle's own weights."""
import math

import numpy as np
import pytest
from scipy.special import softmax

import synth_inputs as S


def test_integer_weights_follow_two_to_the_t(oracle):
    """E_v = trunc(2^t * 2^30) up to the polynomial's 1.4e-7 relative error, t = (y - max) * log2 e."""
    g = np.random.default_rng(1)
    z = np.concatenate([[0.0], -g.random(4000) * 24.0, [-21.5, -30.0, -31.1, -40.0, -1e4]]).astype(np.float32)
    E, Ssum = oracle.logit_weights(z)
    assert E[0] == 1 << 30 and Ssum == int(E.sum())
    for v in range(len(z)):
        t = (float(z[v]) - 0.0) * math.log2(math.e)
        want = 2.0 ** t * (1 << 30)
        assert abs(int(E[v]) - want) <= 3e-7 * want + 1.0 + 2e-6 * abs(t) * want, (v, z[v], E[v], want)
    assert E[-1] == 0 and E[-2] == 0              # far below 2^-30 of the maximum: exactly zero
    assert (np.diff(E[np.argsort(-z)].astype(np.int64)) <= 0).all()   # monotone in the logit


@pytest.mark.parametrize("inv_temp", [1.0, 0.7, 2.5])
def test_normalised_weights_are_softmax(oracle, inv_temp):
    g = np.random.default_rng(2)
    z = g.normal(0, 2, 5000).astype(np.float32)
    E, Ssum = oracle.logit_weights(z, inv_temp)
    ref = softmax(z.astype(np.float64) * np.float64(np.float32(inv_temp)))
    # truncation loses at most one unit per token (V / S in total), the polynomial 1.4e-7 relative
    assert np.abs(E.astype(np.float64) / Ssum - ref).sum() < 2.0 * len(z) / Ssum + 5e-7
    zb = S.f32_to_bf16_bits(z)
    Eb, Sb = oracle.logit_weights(zb, inv_temp)
    refb = softmax(S.bf16_bits_to_f32(zb).astype(np.float64) * np.float64(np.float32(inv_temp)))
    assert np.abs(Eb.astype(np.float64) / Sb - refb).sum() < 2.0 * len(z) / Sb + 5e-7


def test_power_of_two_rescaling_changes_nothing(oracle):
    """(2z, inv_temp/2) is the same input as (z, inv_temp): y = z * inv_temp is formed exactly the same."""
    cfg = S.CONFIGS["C1"].with_(B=64, V=777, k=3)
    g = np.random.default_rng(3)
    zt = g.normal(0, 2, (cfg.B, cfg.k + 1, cfg.V)).astype(np.float32)
    zd = (zt[:, :cfg.k] + g.normal(0, 0.7, (cfg.B, cfg.k, cfg.V))).astype(np.float32)
    draft = g.integers(0, cfg.V, (cfg.B, cfg.k)).astype(np.int32)
    u = (g.integers(0, 1 << 24, (cfg.B, cfg.k + 1)) / float(1 << 24)).astype(np.float32)
    a = oracle.spec_accept_logits(zt, zd, draft, u, 1.0)
    b = oracle.spec_accept_logits(2 * zt, 2 * zd, draft, u, 0.5)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_greedy_limit(oracle):
    """A huge inverse temperature makes both distributions one-hot: exactly the longest matching
    prefix is accepted and the next token is the target's arg-max."""
    V, k, N = 50, 3, 400
    g = np.random.default_rng(4)
    zt = g.normal(0, 1, (N, k + 1, V)).astype(np.float32)
    zd = g.normal(0, 1, (N, k, V)).astype(np.float32)
    zd[::2] = zt[::2, :k]                                  # half the branches: the draft agrees everywhere
    zd[1::4, 1] = -zt[1::4, 1]
    draft = zd.argmax(-1).astype(np.int32)                 # greedy draft
    u = g.random((N, k + 1)).astype(np.float32)
    n, t = oracle.spec_accept_logits(zt, zd, draft, u, 1.0e4)
    ta = zt.argmax(-1)
    for b in range(N):
        want = 0
        while want < k and ta[b, want] == draft[b, want]:
            want += 1
        assert n[b] == want and t[b] == ta[b, want]
    assert (n[::2] == k).all() and n.min() == 0


@pytest.mark.parametrize("k", [1, 3])
def test_lossless_monte_carlo(oracle, k):
    V, N = 8, 400_000
    g = np.random.default_rng(20 + k)
    zt1 = g.normal(0, 1.5, (k + 1, V)).astype(np.float32)
    zd1 = g.normal(0, 1.5, (k, V)).astype(np.float32)
    p1 = softmax(zt1.astype(np.float64), -1)
    q1 = softmax(zd1.astype(np.float64), -1)
    draft = np.stack([g.choice(V, size=N, p=q1[j]) for j in range(k)], 1).astype(np.int32)
    u = (g.integers(0, 1 << 24, size=(N, k + 1)) / float(1 << 24)).astype(np.float32)
    zt = np.ascontiguousarray(np.broadcast_to(zt1, (N, k + 1, V)))
    zd = np.ascontiguousarray(np.broadcast_to(zd1, (N, k, V)))
    n, t = oracle.spec_accept_logits(zt, zd, draft, u)
    alpha0 = np.minimum(p1[0], q1[0]).sum()
    assert abs((n >= 1).mean() - alpha0) < 4.5 * np.sqrt(alpha0 * (1 - alpha0) / N)
    for j in range(k + 1):
        reached = n >= j
        emitted = np.where(n > j, draft[:, min(j, k - 1)], t)[reached]
        cnt = np.bincount(emitted, minlength=V).astype(np.float64)
        M = cnt.sum()
        chi2 = ((cnt - M * p1[j]) ** 2 / (M * p1[j])).sum()
        assert chi2 < 35.0, (j, chi2)


def test_agrees_with_the_probability_path(oracle):
    """Same decisions as the probability-input oracle fed with softmax(z): the two quantise
    differently, so only knife-edge cases may differ."""
    cfg = S.CONFIGS["C2"].with_(B=600, V=3000, k=4)
    g = S.rng_for(9, 1)
    zt = (g.standard_normal((cfg.B, cfg.k + 1, cfg.V)) * 2).astype(np.float32)
    zd = (zt[:, :cfg.k] + g.standard_normal((cfg.B, cfg.k, cfg.V)) * 0.5).astype(np.float32)
    p = softmax(zt.astype(np.float64), -1).astype(np.float32)
    q = softmax(zd.astype(np.float64), -1).astype(np.float32)
    draft = np.stack([[min(int(np.searchsorted(np.cumsum(q[b, j].astype(np.float64)), g.random())), cfg.V - 1)
                       for j in range(cfg.k)] for b in range(cfg.B)]).astype(np.int32)
    u = (g.integers(0, 1 << 24, (cfg.B, cfg.k + 1)) / float(1 << 24)).astype(np.float32)
    n1, t1 = oracle.spec_accept_logits(zt, zd, draft, u)
    n0, t0 = oracle.spec_accept(p, q, draft, u)
    assert (n1 == n0).mean() >= 0.998
    same = n1 == n0
    assert (t1[same] == t0[same]).mean() >= 0.995
    assert 0.5 < (n1 / cfg.k).mean() < 0.95


def test_decisions_recomputed_with_python_integers(oracle):
    """Take the oracle's own integer weights and redo the accept test, the residual and the
    inverse CDF with Python's unbounded integers."""
    V, k, N = 40, 3, 300
    g = np.random.default_rng(6)
    zt = g.normal(0, 2, (N, k + 1, V)).astype(np.float32)
    zd = (zt[:, :k] + g.normal(0, 1.0, (N, k, V))).astype(np.float32)
    zd[:20] = zt[:20, :k]                                  # identical rows: the empty-residual fallback is reachable
    zt[5:10, :, 3] = -1e5
    draft = g.integers(0, V, (N, k)).astype(np.int32)
    draft[5:10, 0] = 3                                     # a draft token the target gives no weight at all
    u = (g.integers(0, 1 << 24, (N, k + 1)) / float(1 << 24)).astype(np.float32)
    u[:20, :k] = np.float32(1.0) - np.float32(2.0 ** -24)   # as close to a rejection as a uniform gets
    n, t = oracle.spec_accept_logits(zt, zd, draft, u, 0.9)
    for b in range(N):
        want_n = 0
        Ep = Eq = None
        Sp = Sq = 0
        for j in range(k):
            Ep, Sp = oracle.logit_weights(zt[b, j], 0.9)
            Eq, Sq = oracle.logit_weights(zd[b, j], 0.9)
            U = int(u[b, j] * (1 << 24))
            x = draft[b, j]
            if U * int(Eq[x]) * Sp < (1 << 24) * int(Ep[x]) * Sq:
                want_n += 1
            else:
                break
        assert n[b] == want_n
        if want_n < k:
            W = [max(0, int(Ep[v]) * Sq - int(Eq[v]) * Sp) for v in range(V)]
            if sum(W) == 0:
                W = [int(e) for e in Ep]
        else:
            Ep, Sp = oracle.logit_weights(zt[b, k], 0.9)
            W = [int(e) for e in Ep]
        T = (int(u[b, k] * (1 << 24)) * sum(W)) >> 24
        run, want_t = 0, -1
        for v in range(V):
            run += W[v]
            if run > T:
                want_t = v
                break
        assert t[b] == want_t
    assert (n[5:10] == 0).all()


def test_rollback_keeps_exactly_the_verified_tokens(oracle):
    """priv_len comes in counting the k + 1 new tokens (last emitted token + k drafts) and goes out counting the
    tokens whose keys and values stay valid: the old cache, the last emitted token and the n accepted drafts.
    Over a run of steps the cache therefore grows by exactly the tokens emitted (n + 1 per step)."""
    V, k, B, steps = 60, 4, 50, 6
    g = np.random.default_rng(12)
    cache = g.integers(0, 500, B).astype(np.int32)          # valid private tokens before the first step
    start = cache.copy()
    emitted = np.zeros(B, np.int64)
    seen = set()
    for _ in range(steps):
        zt = g.normal(0, 2, (B, k + 1, V)).astype(np.float32)
        zd = (zt[:, :k] + g.normal(0, 0.8, (B, k, V))).astype(np.float32)
        draft = np.stack([[g.choice(V, p=softmax(zd[b, j].astype(np.float64))) for j in range(k)]
                          for b in range(B)]).astype(np.int32)
        u = (g.integers(0, 1 << 24, (B, k + 1)) / float(1 << 24)).astype(np.float32)
        pl = (cache + k + 1).astype(np.int32)                # what the attention of this step is given
        n, t = oracle.spec_accept_logits(zt, zd, draft, u, priv_len=pl)
        n0, t0 = oracle.spec_accept_logits(zt, zd, draft, u)
        assert np.array_equal(n, n0) and np.array_equal(t, t0)   # the bookkeeping changes no decision
        assert np.array_equal(pl, cache + 1 + n)
        cache = pl
        emitted += n + 1
        seen.update(n.tolist())
    assert np.array_equal(cache - start, emitted)
    assert seen == set(range(k + 1))                         # every acceptance length occurred


def test_rows_without_any_weight_give_no_token(oracle):
    """A softmax over logits that are all -inf has no mass: every integer weight is 0.  A draft at such a target
    row cannot be accepted (its probability is 0), nothing can be sampled there, and the token is -1 -- the same
    convention as the probability path, which returns -1 for a row of zeros."""
    V, k = 40, 2
    g = np.random.default_rng(21)
    zt = g.normal(0, 2, (3, k + 1, V)).astype(np.float32)
    zd = zt[:, :k].copy()                                    # identical rows: drafts are accepted wherever they weigh
    zt[1, 1, :] = -np.inf                                    # branch 1: no mass at position 1
    zt[2, 2, :] = -np.inf                                    # branch 2: no mass at the bonus position
    E, S = oracle.logit_weights(zt[1, 1])
    assert S == 0 and not E.any()
    draft = np.array([[3, 4], [5, 6], [7, 8]], np.int32)
    u = np.full((3, k + 1), 0.25, np.float32)
    n, t = oracle.spec_accept_logits(zt, zd, draft, u)
    assert list(n) == [2, 1, 2] and t[0] >= 0 and t[1] == -1 and t[2] == -1
    # the probability path on the corresponding distributions (zeros where there is no mass) agrees
    p = softmax(zt.astype(np.float64), axis=-1)
    p[1, 1, :] = 0.0
    p[2, 2, :] = 0.0
    q = softmax(zd.astype(np.float64), axis=-1)
    n2, t2 = oracle.spec_accept(p.astype(np.float32), q.astype(np.float32), draft, u)
    assert list(n2) == [2, 1, 2] and t2[1] == -1 and t2[2] == -1
