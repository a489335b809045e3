/*
 * CPU oracle for the speculative verification step across B reasoning branches.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU library is
 * checked against.  It shares no code, header, table or helper with the HIP path, and the
 * product never calls it: only the tests, the smoke check and the bench's cpu-baseline leg
 * may load it.
 *
 * What it follows in the paper ("Faster and Better LLMs via Latency-Aware Test-Time
 * Scaling", arXiv 2505.19634):
 *   - Section 3.2, branch-wise parallelism: B concurrent branches of one question, the
 *     question's prompt being common to all of them, aggregated by majority voting.
 *   - Section 3.2, sequence-wise parallelism, and Section 2 (speculative decoding): a draft
 *     model proposes gamma (= k) tokens, the target model verifies them in one parallel
 *     forward, losslessly.  The acceptance rule itself is the one of the works the paper
 *     cites for it (Leviathan et al. 2023; Chen et al. 2023): accept draft x with
 *     probability min(1, p(x)/q(x)); on the first rejection draw from
 *     norm(max(0, p - q)); if all k are accepted draw the bonus token from p_k.
 *   - Section 3.1: decoding is bound by loading weights and KV caches; the attention of
 *     the k + 1 new positions over the branch's KV cache is the part computed here.
 *
 * All floating point is fp64 on the stored input values (bf16 / fp32 inputs convert to
 * fp64 exactly).  Loops are in definition order; OpenMP only distributes independent
 * outputs over threads.
 *
 * Pins (tests/test_oracle_*.py): brute-force softmax(QK^T/sqrt d)V on tiny shapes, closed
 * forms (Q = 0, one-hot limit), k = 0 == decode attention, prefix-boundary invariance,
 * causality; greedy == longest matching prefix, Monte-Carlo losslessness, closed-form
 * acceptance probability, exhaustive fixed-point sampler counts; O(B^2) vote brute force.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static double load_elem(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    /* bfloat16 = upper 16 bits of an IEEE fp32 */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/*
 * Causal attention of the R = k + 1 new rows of every branch (Section 3.2 / Section 2:
 * the target model's parallel verification of the drafts).
 *
 * Layouts (dense, row-major):
 *   Q     [B][R][Hq][D]
 *   Kpre  [Hkv][P][D], Vpre likewise     -- the prompt's KV, one copy for all branches
 *   Kpriv [B][Hkv][Lmax][D], Vpriv likewise
 *   priv_len [B]: private tokens of branch b, the last R of which are the new tokens
 *   O     [B][R][Hq][D] fp64,  lse [B][R][Hq] fp64 (natural log), may be NULL
 * Query head h reads KV head h / (Hq / Hkv).  Row i of branch b sees the P prefix keys and
 * the first priv_len[b] - k + i private keys (itself included, later drafts excluded).
 * scale <= 0 selects 1 / sqrt(D).
 * Returns 0, or -1 on a malformed call.
 */
int oracle_verify_attention(int B, int k, int Hq, int Hkv, int D, int P, int Lmax, int dtype,
                            double scale, const void *Q, const void *Kpre, const void *Vpre,
                            const void *Kpriv, const void *Vpriv, const int32_t *priv_len,
                            double *O, double *lse)
{
    if (B < 1 || k < 0 || Hq < 1 || Hkv < 1 || Hq % Hkv || D < 1 || P < 0 || Lmax < k + 1)
        return -1;
    const int R = k + 1, G = Hq / Hkv;
    if (scale <= 0.0)
        scale = 1.0 / sqrt((double)D);
    int status = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const int Lb = priv_len[b];
            if (Lb < R || Lb > Lmax) {
                status = -1;
                continue;
            }
            double *s = (double *)malloc(sizeof(double) * (size_t)(P + Lb));
            for (int i = 0; i < R; ++i) {
                const int n_priv = Lb - k + i;    /* visible private keys of row i */
                const int n = P + n_priv;
                const int64_t qoff = (((int64_t)b * R + i) * Hq + h) * D;
                /* scores */
                for (int j = 0; j < n; ++j) {
                    const void *Kb;
                    int64_t koff;
                    if (j < P) {
                        Kb = Kpre;
                        koff = ((int64_t)g * P + j) * D;
                    } else {
                        Kb = Kpriv;
                        koff = (((int64_t)b * Hkv + g) * Lmax + (j - P)) * D;
                    }
                    double acc = 0.0;
                    for (int d = 0; d < D; ++d)
                        acc += load_elem(Q, dtype, qoff + d) * load_elem(Kb, dtype, koff + d);
                    s[j] = acc * scale;
                }
                /* softmax with the maximum subtracted */
                double mx = s[0];
                for (int j = 1; j < n; ++j)
                    if (s[j] > mx)
                        mx = s[j];
                double denom = 0.0;
                for (int j = 0; j < n; ++j) {
                    s[j] = exp(s[j] - mx);
                    denom += s[j];
                }
                /* weighted sum of values */
                for (int d = 0; d < D; ++d) {
                    double acc = 0.0;
                    for (int j = 0; j < n; ++j) {
                        const void *Vb;
                        int64_t voff;
                        if (j < P) {
                            Vb = Vpre;
                            voff = ((int64_t)g * P + j) * D;
                        } else {
                            Vb = Vpriv;
                            voff = (((int64_t)b * Hkv + g) * Lmax + (j - P)) * D;
                        }
                        acc += s[j] * load_elem(Vb, dtype, voff + d);
                    }
                    O[qoff + d] = acc / denom;
                }
                if (lse)
                    lse[((int64_t)b * R + i) * Hq + h] = mx + log(denom);
            }
            free(s);
        }
    }
    return status;
}

/*
 * Fixed-point weight of one residual value: trunc(r * 2^40) with the product formed in
 * fp32 (scaling by a power of two is exact there, r <= 1 so there is no overflow).
 * Anything below 2^-40, every denormal included, becomes 0.
 */
static uint64_t fixed_weight(float r)
{
    float scaled = r * 1099511627776.0f; /* 2^40 */
    return (uint64_t)scaled;             /* C conversion truncates toward zero */
}

static float residual_value(const float *prow, const float *qrow, int v)
{
    if (qrow == NULL)
        return prow[v];
    float r = prow[v] - qrow[v]; /* one IEEE fp32 subtraction */
    return r > 0.0f ? r : 0.0f;
}

/*
 * Speculative-sampling acceptance for B independent branches (rule of the works cited in
 * Section 2 and Section 3.2 for lossless speculative decoding).
 *
 *   p [B][k+1][V] target distributions at draft positions 0..k-1 and the bonus position k
 *   q [B][k][V]   draft distributions (NULL iff k == 0)
 *   draft [B][k]  draft tokens, each in [0, V)
 *   u [B][k+1]    uniforms in [0, 1): u[b][j] decides draft j, u[b][k] drives the sample
 *   accept_len [B] out: drafts accepted before the first rejection
 *   next_token [B] out: the resampled token (rejection) or the bonus token (all accepted);
 *                       -1 iff the row to sample carries no mass at all
 *
 * The draw is made on an integer fixed-point CDF so that it does not depend on summation
 * order: w_v = trunc(r_v * 2^40), Z = sum w_v, threshold T = floor(m * Z / 2^24) with
 * m = trunc(u * 2^24); the token is the first v whose inclusive prefix sum exceeds T.
 * Returns 0, or -1 on a malformed call.
 */
int oracle_spec_accept(int B, int k, int V, const float *p, const float *q, const int32_t *draft,
                       const float *u, int32_t *accept_len, int32_t *next_token)
{
    if (B < 1 || k < 0 || V < 1 || !p || !u || !accept_len || !next_token || (k > 0 && (!q || !draft)))
        return -1;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const float *pb = p + (int64_t)b * (k + 1) * V;
        const float *qb = q ? q + (int64_t)b * k * V : NULL;
        const float *ub = u + (int64_t)b * (k + 1);
        /* accept drafts in order while u < min(1, p(x)/q(x)), i.e. u*q(x) < p(x);
           the product of two fp32 values is exact in fp64, so this is the exact test */
        int n = 0;
        for (int j = 0; j < k; ++j) {
            const int x = draft[(int64_t)b * k + j];
            if (x < 0 || x >= V) {
                status = -1;
                break;
            }
            const double pv = (double)pb[(int64_t)j * V + x];
            const double qv = (double)qb[(int64_t)j * V + x];
            const double uv = (double)ub[j];
            if (uv * qv < pv)
                ++n;
            else
                break;
        }
        accept_len[b] = n;
        /* the row to sample: residual of position n after a rejection, else the bonus row */
        const float *prow = pb + (int64_t)n * V;
        const float *qrow = (n < k) ? qb + (int64_t)n * V : NULL;
        uint64_t Z = 0;
        for (int v = 0; v < V; ++v)
            Z += fixed_weight(residual_value(prow, qrow, v));
        if (Z == 0 && qrow) { /* degenerate residual (p == q everywhere): fall back to p */
            qrow = NULL;
            for (int v = 0; v < V; ++v)
                Z += fixed_weight(residual_value(prow, qrow, v));
        }
        if (Z == 0) {
            next_token[b] = -1;
            continue;
        }
        const uint32_t m = (uint32_t)(ub[k] * 16777216.0f); /* trunc(u * 2^24) */
        const uint64_t T = (uint64_t)(((unsigned __int128)m * (unsigned __int128)Z) >> 24);
        uint64_t run = 0;
        int tok = -1;
        for (int v = 0; v < V; ++v) {
            run += fixed_weight(residual_value(prow, qrow, v));
            if (run > T) {
                tok = v;
                break;
            }
        }
        next_token[b] = tok;
    }
    return status;
}

/*
 * Majority voting over the branches' final answers (Section 1 / Section 4.1: the answer
 * given by most branches wins).  answers [N][B]; ids < 0 mean "no answer" and are not
 * counted.  Ties go to the id that occurs first (smallest branch index).  All excluded:
 * winner -1, count 0.
 */
int oracle_majority_vote(int N, int B, const int32_t *answers, int32_t *winner, int32_t *winner_count)
{
    if (N < 1 || B < 1 || !answers || !winner || !winner_count)
        return -1;
    for (int n = 0; n < N; ++n) {
        const int32_t *a = answers + (int64_t)n * B;
        int32_t best = -1, best_count = 0;
        for (int i = 0; i < B; ++i) {
            if (a[i] < 0)
                continue;
            int32_t c = 0;
            for (int j = 0; j < B; ++j)
                if (a[j] == a[i])
                    ++c;
            if (c > best_count) { /* strict: an earlier id keeps a tie */
                best = a[i];
                best_count = c;
            }
        }
        winner[n] = best;
        winner_count[n] = best_count;
    }
    return 0;
}
