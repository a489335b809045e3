"""Pins for the majority-vote oracle: a counting dictionary, hand cases, invariants."""
from collections import Counter

import numpy as np

import synth_inputs as S


def by_counter(row):
    c = Counter(int(a) for a in row if a >= 0)
    if not c:
        return -1, 0
    top = max(c.values())
    for a in row:                       # first occurrence among the tied ids
        if a >= 0 and c[int(a)] == top:
            return int(a), top


def test_hand_cases(oracle):
    cases = [([3], (3, 1)), ([5, 5, 5, 5], (5, 4)), ([1, 2, 2, 1], (1, 2)), ([2, 1, 1, 2], (2, 2)),
             ([-1, -1], (-1, 0)), ([-1, 7, -1], (7, 1)), ([4, -1, 9, 9, 4, 9], (9, 3)), ([0, 1, 2, 3], (0, 1))]
    for row, want in cases:
        w, c = oracle.majority_vote(np.array(row, np.int32))
        assert (int(w[0]), int(c[0])) == want, row


def test_against_counting_dictionary_on_zipf_answers(oracle):
    cfg = S.CONFIGS["C3"]
    ties = 0
    for salt in range(40):
        a = S.vote_inputs(cfg, N=25, salt=salt)
        a[::7, ::5] = -1
        w, c = oracle.majority_vote(a)
        for n in range(a.shape[0]):
            want = by_counter(a[n])
            assert (int(w[n]), int(c[n])) == want
            cnt = Counter(int(x) for x in a[n] if x >= 0)
            ties += sum(1 for v in cnt.values() if v == want[1]) > 1
    assert ties > 20                     # the tie-break really is exercised


def test_permutation_invariance(oracle):
    g = np.random.default_rng(3)
    for _ in range(200):
        a = g.integers(0, 6, size=16).astype(np.int32)
        w0, c0 = oracle.majority_vote(a)
        a2 = g.permutation(a)
        w1, c1 = oracle.majority_vote(a2)
        assert c0[0] == c1[0]            # the winning count never depends on branch order
        cnt = Counter(a.tolist())
        if sum(1 for v in cnt.values() if v == c0[0]) == 1:
            assert w0[0] == w1[0]        # nor does the winner when it is unique
