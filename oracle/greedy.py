"""Oracle of the search for the latency-optimal configuration (paper Algorithm 1, Section 3.3).
Test infrastructure only.

The search is a hill climb on the lattice of configurations (B, gamma) with B a power of two:
from (1, 0), a configuration has at most two successors -- twice the branches, or one more draft
token -- and the climb moves to the successor with the higher accuracy while that is a strict
improvement.  `tts_task(B, gamma, T)` is the accuracy reached under the latency budget T.
Returns (B, gamma, acc, rounds, evaluations); `rounds` counts every visit of a configuration at
which successors were looked at (or found to be out of bounds), the last one included: the
"steps" column of the paper's grid-vs-greedy table.
"""


def greedy_search(tts_task, T, B_max=None, gamma_max=None):
    def successors(cfg):
        """In order of preference: max() below returns the first of equal accuracies, so the
        branch move wins a tie."""
        B, gamma = cfg
        out = []
        if B_max is None or 2 * B <= B_max:
            out.append((2 * B, gamma))
        if gamma_max is None or gamma + 1 <= gamma_max:
            out.append((B, gamma + 1))
        return out

    here = (1, 0)
    acc_here = tts_task(1, 0, T)
    evaluations, rounds = 1, 0
    climbing = True
    while climbing:
        rounds += 1
        scored = [(tts_task(B, gamma, T), (B, gamma)) for B, gamma in successors(here)]
        evaluations += len(scored)
        climbing = False
        if scored:
            acc_best, best = max(scored, key=lambda entry: entry[0])
            if acc_best > acc_here:
                here, acc_here, climbing = best, acc_best, True
    return here[0], here[1], acc_here, rounds, evaluations
