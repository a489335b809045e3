"""Pins for the confidence-weighted aggregation oracle: hand cases from the definitions in the
paper's aggregation ablation, a dictionary-based re-computation, and reductions to majority voting."""
from collections import OrderedDict

import numpy as np

import synth_inputs as S


def q30(c):
    return int(np.float32(c) * np.float32(2.0 ** 30))


def by_dict(answers, conf, lens, wmode, smode):
    w = {}
    for b, a in enumerate(answers):
        if a < 0 or lens[b] <= 0:
            continue
        qs = [q30(c) for c in conf[b][:lens[b]]]
        w[b] = np.float32(min(qs) / 2.0 ** 30) if wmode == "min" else np.float32(sum(qs) / (len(qs) * 2.0 ** 30))
    if not w:
        return -1, np.float32(0)
    if smode == "max":
        best = max(w.values())
        b = min(b for b in w if w[b] == best)
        return int(answers[b]), best
    score = OrderedDict()
    for b in w:                                  # branch order
        score[answers[b]] = np.float32(score.get(answers[b], np.float32(0)) + w[b])
    best = max(score.values())
    for a, s in score.items():                   # insertion order = first occurrence
        if s == best:
            return int(a), s


def test_hand_cases(oracle):
    answers = np.array([[7, 3, 7, 5]], np.int32)
    conf = np.array([[[0.9, 0.2], [0.6, 0.7], [0.5, 0.4], [0.95, 0.95]]], np.float32)
    # min weights: .2 .6 .4 .95   avg weights: .55 .65 .45 .95
    assert oracle.confidence_vote(answers, conf, None, "min", "max")[0][0] == 5
    assert oracle.confidence_vote(answers, conf, None, "avg", "max")[0][0] == 5
    w, s = oracle.confidence_vote(answers, conf, None, "avg", "vote")       # 7: 1.0, 3: .65, 5: .95
    assert w[0] == 7 and abs(s[0] - 1.0) < 1e-6
    w, s = oracle.confidence_vote(answers, conf, None, "min", "vote")       # 7: .6, 3: .6, 5: .95
    assert w[0] == 5
    lens = np.array([[2, 2, 2, 0]], np.int32)                                # branch 3 has no scores: left out
    w, s = oracle.confidence_vote(answers, conf, lens, "min", "vote")       # 7: .6 (first), 3: .6
    assert w[0] == 7
    w, s = oracle.confidence_vote(np.array([[-1, -1]], np.int32), conf[:, :2], None, "avg", "vote")
    assert w[0] == -1 and s[0] == 0


def test_against_dictionary(oracle):
    g = np.random.default_rng(8)
    cfg = S.CONFIGS["C3"]
    for trial in range(60):
        B, T = 16, 37
        answers = S.vote_inputs(cfg, N=1, salt=trial)[0]
        answers[g.random(B) < 0.1] = -1
        conf = (0.3 + 0.7 * g.random((B, T))).astype(np.float32)
        lens = g.integers(0, T + 1, B).astype(np.int32)
        for wm in ("min", "avg"):
            for sm in ("max", "vote"):
                w, s = oracle.confidence_vote(answers[None], conf[None], lens[None], wm, sm)
                want = by_dict(answers, conf, lens, wm, sm)
                assert int(w[0]) == want[0] and s[0] == want[1], (trial, wm, sm)


def test_equal_confidences_reduce_to_majority_voting(oracle):
    cfg = S.CONFIGS["C3"]
    for salt in range(30):
        a = S.vote_inputs(cfg, N=5, salt=100 + salt)
        conf = np.full((5, cfg.B, 4), 0.5, np.float32)
        w, s = oracle.confidence_vote(a, conf, None, "avg", "vote")
        w0, c0 = oracle.majority_vote(a)
        assert np.array_equal(w, w0)
        assert np.allclose(s, 0.5 * c0)
