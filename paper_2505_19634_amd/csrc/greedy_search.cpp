// greedy_search: the configuration search of the paper's Algorithm 1 -- host code, no GPU work.
// Starting from one branch and no draft tokens, each round evaluates doubling the branches and
// adding one draft token, moves to the better of the two (branches on a tie) if that improves the
// accuracy, and stops otherwise; O((log2 B* + 1) + gamma*) rounds instead of the grid's
// (log2 B_max + 1) * (gamma_max + 1) evaluations (Section 3.3).
#include "lotts.h"

extern "C" int greedy_search(lotts_tts_task_fn tts_task, void* user, double T, int32_t B_max, int32_t gamma_max,
                             int32_t* B_opt, int32_t* gamma_opt, double* acc_opt, int32_t* rounds,
                             int32_t* evaluations) {
    if (!tts_task || !B_opt || !gamma_opt || !acc_opt) return LOTTS_ERR_NULL;
    if (B_max < 1 || gamma_max < 0 || B_max > (1 << 30)) return LOTTS_ERR_SHAPE;
    int32_t B = 1, gamma = 0, n_rounds = 0, n_evals = 1;
    double acc = tts_task(B, gamma, T, user);
    for (;;) {
        ++n_rounds;
        const bool can_b = 2 * (int64_t)B <= B_max, can_g = gamma + 1 <= gamma_max;
        if (!can_b && !can_g) break;
        double acc_b = 0.0, acc_g = 0.0;
        if (can_b) {
            acc_b = tts_task(2 * B, gamma, T, user);
            ++n_evals;
        }
        if (can_g) {
            acc_g = tts_task(B, gamma + 1, T, user);
            ++n_evals;
        }
        const bool take_b = can_b && (!can_g || acc_b >= acc_g);
        const double acc_new = take_b ? acc_b : acc_g;
        if (!(acc_new > acc)) break;
        if (take_b) B *= 2; else gamma += 1;
        acc = acc_new;
    }
    *B_opt = B;
    *gamma_opt = gamma;
    *acc_opt = acc;
    if (rounds) *rounds = n_rounds;
    if (evaluations) *evaluations = n_evals;
    return LOTTS_OK;
}
