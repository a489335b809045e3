"""Oracle of the greedy (B, gamma) search (paper Algorithm 1).  Test infrastructure only.

Start from one branch and no drafts; each round evaluate doubling the branches and adding one
draft token, keep the better of the two (branches on a tie) if it improves the accuracy, stop
otherwise.  `tts_task(B, gamma, T)` returns the accuracy reached under latency budget T.
Returns (B, gamma, acc, rounds, evaluations): rounds counts the iterations of the loop, the
terminating one included -- the "steps" of the paper's grid-vs-greedy table.
"""


def greedy_search(tts_task, T, B_max=None, gamma_max=None):
    B, gamma = 1, 0
    acc = tts_task(B, gamma, T)
    evals, rounds = 1, 0
    while True:
        rounds += 1
        acc_b = acc_g = None
        if B_max is None or 2 * B <= B_max:
            acc_b = tts_task(2 * B, gamma, T)
            evals += 1
        if gamma_max is None or gamma + 1 <= gamma_max:
            acc_g = tts_task(B, gamma + 1, T)
            evals += 1
        if acc_b is None and acc_g is None:
            break
        if acc_g is None or (acc_b is not None and acc_b >= acc_g):
            B_new, g_new, acc_new = 2 * B, gamma, acc_b
        else:
            B_new, g_new, acc_new = B, gamma + 1, acc_g
        if acc_new > acc:
            B, gamma, acc = B_new, g_new, acc_new
        else:
            break
    return B, gamma, acc, rounds, evals
