"""Greedy (B, gamma) search of Algorithm 1: the oracle against the paper's printed step counts,
then the library's host function against the oracle.  No GPU involved."""
import itertools
import math
import os
import re

import numpy as np
import pytest

from oracle.greedy import greedy_search as oracle_greedy

HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_values.txt")):
        m = re.match(r"\s*([A-Za-z_0-9]+)\s*=\s*([0-9.e+-]+)", line)
        if m:
            out[m.group(1)] = float(m.group(2))
    return out


def peaked(B_star, g_star):
    """An accuracy surface with a single optimum at (B*, gamma*), separable and strictly unimodal
    along both moves; the branch move is worth more than the draft move at equal distance."""
    def task(B, gamma, T):
        return 0.9 - 0.03 * abs(math.log2(B) - math.log2(B_star)) - 0.02 * abs(gamma - g_star)
    return task


@pytest.mark.parametrize("B_star,g_star", [(16, 5), (32, 5), (16, 4), (4, 5)])
def test_oracle_reproduces_the_papers_step_counts(B_star, g_star):
    g = golden()
    B, gamma, acc, rounds, evals = oracle_greedy(peaked(B_star, g_star), 60.0, 64, 7)
    assert (B, gamma) == (B_star, g_star)
    assert rounds == g["greedy_steps_B%d_g%d" % (B_star, g_star)] == math.log2(B_star) + 1 + g_star
    assert abs(acc - 0.9) < 1e-12
    assert evals == 1 + 2 * rounds
    assert g["grid_steps"] == len(list(itertools.product(range(7), range(8))))


def test_oracle_finds_the_grid_optimum_on_unimodal_surfaces():
    rng = np.random.default_rng(0)
    for _ in range(200):
        B_star, g_star = 2 ** int(rng.integers(0, 7)), int(rng.integers(0, 8))
        task = peaked(B_star, g_star)
        grid = max(((task(2 ** i, j, 0), -i, -j) for i in range(7) for j in range(8)))
        B, gamma, acc, rounds, _ = oracle_greedy(task, 0.0, 64, 7)
        assert acc == grid[0] and (B, gamma) == (B_star, g_star)
        assert rounds == math.log2(B_star) + g_star + (0 if (B_star == 64 and g_star == 7) else 1) or \
            rounds == math.log2(B_star) + g_star + 1


def test_oracle_rules():
    # a tie between the two moves goes to the branch move
    assert oracle_greedy(lambda B, g, T: 0.5 + 0.1 * (B > 1) + 0.1 * (g > 0) - 0.2 * (B > 1 and g > 0) - 1.0 * (B > 2 or g > 1),
                         1.0, 64, 7)[:2] == (2, 0)
    # no strict improvement: stay at the baseline after one round of two evaluations
    assert oracle_greedy(lambda B, g, T: 0.7, 1.0, 64, 7) == (1, 0, 0.7, 1, 3)
    # bounds are respected and not evaluated beyond
    seen = []

    def rising(B, g, T):
        seen.append((B, g))
        return B + g
    assert oracle_greedy(rising, 1.0, 4, 1)[:2] == (4, 1)
    assert all(B <= 4 and g <= 1 for B, g in seen)


def test_library_matches_the_oracle():
    import paper_2505_19634_amd as lotts
    rng = np.random.default_rng(1)
    for trial in range(300):
        table = rng.random((8, 9))                      # arbitrary (not unimodal) accuracy tables
        if trial % 3 == 0:
            table = np.round(table, 1)                  # with ties
        task = lambda B, g, T: float(table[int(math.log2(B)), g])
        Bm, gm = 2 ** int(rng.integers(0, 7)), int(rng.integers(0, 8))
        assert lotts.greedy_search(task, 30.0, Bm, gm) == oracle_greedy(task, 30.0, Bm, gm)
    for B_star, g_star in [(16, 5), (32, 5), (16, 4), (4, 5)]:
        assert lotts.greedy_search(peaked(B_star, g_star), 60.0)[:2] == (B_star, g_star)
    with pytest.raises(lotts.LottsError):
        lotts.greedy_search(lambda B, g, T: 0.0, 1.0, 0, 3)
