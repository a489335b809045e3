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

/* =====================================================================================
 * Widening 1: acceptance straight from logits (no materialised p, q).
 *
 * The distributions are softmax(z * inv_temp) of the target / draft logits (Section 2: the
 * draft proposes, the target verifies; the paper states no temperature, so it is an argument).
 * To stay independent of summation order AND of the platform's exp(), the softmax is defined
 * through integers: for a row with y_v = fp32(z_v) * inv_temp and m = max_v y_v,
 *     t_v = (y_v - m) * log2(e)                      two fp32 operations
 *     E_v = trunc( P(frac(-t_v)) * 2^(30 - floor(-t_v)) ),  0 if floor(-t_v) >= 31
 * where P is a fixed degree-6 polynomial for 2^-f on [0,1) evaluated by fused multiply-adds
 * (relative error 1.4e-7), S = sum_v E_v, and the probability of v is E_v / S exactly.
 * Accept draft x iff U * Eq(x) * Sp < 2^24 * Ep(x) * Sq with U = trunc(u * 2^24) (this is
 * u < min(1, p/q) on the rationals); residual weights W_v = max(0, Ep_v * Sq - Eq_v * Sp),
 * bonus weights W_v = Ep_v; token = first v with prefix sum > floor(U_k * sum W / 2^24).
 * 128-bit integers throughout; V <= 2^20.
 * ===================================================================================== */
static float pow2_neg_poly(float f)
{
    /* 2^-f on [0, 1): coefficients fixed by this specification (c0 = 1 exactly) */
    float g = 0x1.e243bep-14f;
    g = fmaf(g, f, -0x1.52a284p-10f);
    g = fmaf(g, f, 0x1.3a7ae4p-7f);
    g = fmaf(g, f, -0x1.c6a66cp-5f);
    g = fmaf(g, f, 0x1.ebfbaap-3f);
    g = fmaf(g, f, -0x1.62e430p-1f);
    g = fmaf(g, f, 1.0f);
    return g;
}

static uint64_t logit_weight(float y, float m)
{
    float t = (y - m) * 0x1.715476p+0f; /* log2(e) */
    float a = -t;
    float nf = floorf(a);
    if (!(nf < 31.0f))
        return 0;
    float f = a - nf;
    float g = pow2_neg_poly(f);
    return (uint64_t)(g * ldexpf(1.0f, 30 - (int)nf));
}

static float logit_at(const void *z, int dtype, int64_t idx, float inv_temp)
{
    return (float)load_elem(z, dtype, idx) * inv_temp;
}

/* Integer softmax weights of one row of V logits (exposed for the tests): E[V], returns S. */
uint64_t oracle_logit_weights(int V, const void *z, int dtype, float inv_temp, uint64_t *E)
{
    float m = logit_at(z, dtype, 0, inv_temp);
    for (int v = 1; v < V; ++v) {
        float y = logit_at(z, dtype, v, inv_temp);
        if (y > m)
            m = y;
    }
    uint64_t S = 0;
    for (int v = 0; v < V; ++v) {
        E[v] = logit_weight(logit_at(z, dtype, v, inv_temp), m);
        S += E[v];
    }
    return S;
}

typedef unsigned __int128 u128;

int oracle_spec_accept_logits(int B, int k, int V, const void *zt, const void *zd, int dtype, float inv_temp,
                              const int32_t *draft, const float *u, int32_t *accept_len, int32_t *next_token,
                              int32_t *priv_len)
{
    if (B < 1 || k < 0 || V < 1 || V > (1 << 20) || !zt || !u || !accept_len || !next_token ||
        (k > 0 && (!zd || !draft)) || !(inv_temp > 0.0f))
        return -1;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        uint64_t *Ep = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)V);
        uint64_t *Eq = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)V);
        const float *ub = u + (int64_t)b * (k + 1);
        const size_t es = dtype == ORACLE_F32 ? 4 : 2;
        uint64_t Sp = 0, Sq = 0;
        int n = 0;
        for (int j = 0; j < k; ++j) {
            const int x = draft[(int64_t)b * k + j];
            if (x < 0 || x >= V) {
                status = -1;
                break;
            }
            Sp = oracle_logit_weights(V, (const char *)zt + ((int64_t)b * (k + 1) + j) * V * es, dtype, inv_temp, Ep);
            Sq = oracle_logit_weights(V, (const char *)zd + ((int64_t)b * k + j) * V * es, dtype, inv_temp, Eq);
            const u128 U = (u128)(uint32_t)(ub[j] * 16777216.0f);
            if (U * Eq[x] * Sp < ((u128)1 << 24) * Ep[x] * Sq)
                ++n;
            else
                break; /* Ep, Eq, Sp, Sq now hold the rows of the rejected position n */
        }
        accept_len[b] = n;
        int have_q = n < k;
        if (!have_q) /* all accepted: the bonus row */
            Sp = oracle_logit_weights(V, (const char *)zt + ((int64_t)b * (k + 1) + k) * V * es, dtype, inv_temp, Ep);
        u128 Z = 0;
        if (have_q) {
            for (int v = 0; v < V; ++v) {
                const u128 a = (u128)Ep[v] * Sq, c = (u128)Eq[v] * Sp;
                Z += a > c ? a - c : 0;
            }
            if (Z == 0)
                have_q = 0; /* identical rows: fall back to the target row */
        }
        if (!have_q)
            Z = Sp;
        uint32_t m24 = (uint32_t)(ub[k] * 16777216.0f);
        const u128 T = ((u128)m24 * Z) >> 24;
        u128 run = 0;
        int tok = -1;
        for (int v = 0; v < V; ++v) {
            if (have_q) {
                const u128 a = (u128)Ep[v] * Sq, c = (u128)Eq[v] * Sp;
                run += a > c ? a - c : 0;
            } else {
                run += Ep[v];
            }
            if (run > T) {
                tok = v;
                break;
            }
        }
        next_token[b] = tok;
        if (priv_len) /* the k - n rejected drafts leave the branch's KV cache */
            priv_len[b] -= k - n;
        free(Ep);
        free(Eq);
    }
    return status;
}

/* =====================================================================================
 * Widening 2: confidence-based aggregation (Section "Different Aggregation Strategies"):
 * every branch's answer is weighted by the minimum or the average of its confidence scores,
 * then either the single most confident answer wins ("max") or the weights of identical
 * answers are added and the largest total wins ("vote").
 *   answers [N][B]; conf [N][B][T] in [0, 1]; conf_len [N][B] valid scores per branch (NULL: T)
 *   weight_mode 0 = min, 1 = avg;  select_mode 0 = max, 1 = vote
 * Branches with id < 0 or without scores do not take part.  Scores are quantised to 2^-30
 * (trunc(c * 2^30)) so that sums are integers: min weight = q_min / 2^30, avg weight =
 * (sum q) / (len * 2^30), both formed in fp64 and rounded once to fp32.  "vote" adds the fp32
 * weights of identical answers in branch order.  Ties go to the earliest branch / earliest
 * first occurrence.  winner = -1, score = 0 if nobody takes part.
 * ===================================================================================== */
int oracle_confidence_vote(int N, int B, int T, const int32_t *answers, const float *conf, const int32_t *conf_len,
                           int weight_mode, int select_mode, int32_t *winner, float *winner_score)
{
    if (N < 1 || B < 1 || T < 1 || !answers || !conf || !winner || !winner_score || weight_mode < 0 ||
        weight_mode > 1 || select_mode < 0 || select_mode > 1)
        return -1;
    for (int n = 0; n < N; ++n) {
        float *w = (float *)malloc(sizeof(float) * (size_t)B);
        int *ok = (int *)malloc(sizeof(int) * (size_t)B);
        for (int b = 0; b < B; ++b) {
            int len = conf_len ? conf_len[(int64_t)n * B + b] : T;
            if (len > T)
                len = T;
            ok[b] = answers[(int64_t)n * B + b] >= 0 && len > 0;
            w[b] = 0.0f;
            if (!ok[b])
                continue;
            const float *c = conf + ((int64_t)n * B + b) * T;
            uint64_t sum = 0, mn = UINT64_MAX;
            for (int t = 0; t < len; ++t) {
                const uint64_t q = (uint64_t)(c[t] * 1073741824.0f); /* trunc(c * 2^30) */
                sum += q;
                if (q < mn)
                    mn = q;
            }
            w[b] = weight_mode == 0 ? (float)((double)mn / 1073741824.0)
                                    : (float)((double)sum / ((double)len * 1073741824.0));
        }
        int32_t best = -1;
        float best_score = 0.0f;
        int have = 0;
        const int32_t *a = answers + (int64_t)n * B;
        for (int i = 0; i < B; ++i) {
            if (!ok[i])
                continue;
            float score;
            if (select_mode == 0) {
                score = w[i];
            } else {
                int first = 1;
                for (int j = 0; j < i; ++j)
                    if (ok[j] && a[j] == a[i])
                        first = 0;
                if (!first)
                    continue;
                score = 0.0f;
                for (int j = 0; j < B; ++j)
                    if (ok[j] && a[j] == a[i])
                        score = score + w[j];
            }
            if (!have || score > best_score) {
                have = 1;
                best = a[i];
                best_score = score;
            }
        }
        winner[n] = best;
        winner_score[n] = have ? best_score : 0.0f;
        free(w);
        free(ok);
    }
    return 0;
}

/* =====================================================================================
 * Widening 3: the weight GEMM of the verify forward.  The target model's forward over the
 * B * (k + 1) new tokens multiplies a skinny activation matrix by every weight matrix, and the
 * weights are what the step loads most of (Section 3.1; Appendix: 64 GB of weights for the 32B
 * model against 0.25 GB of KV cache per branch).
 *   Y[m][n] = sum_k X[m][k] * W[n][k]        X [M][K], W [N][K] (a Linear layer's weight), Y [M][N]
 * bf16 (or fp32) inputs read exactly, fp64 accumulation, fp64 output.
 * ===================================================================================== */
int oracle_skinny_gemm(int M, int N, int K, int dtype, const void *X, const void *W, double *Y)
{
    if (M < 1 || N < 1 || K < 1 || !X || !W || !Y)
        return -1;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += load_elem(X, dtype, (int64_t)m * K + k) * load_elem(W, dtype, (int64_t)n * K + k);
            Y[(int64_t)m * N + n] = acc;
        }
    return 0;
}

/* ---------------------------------------------------------------------------------------------
 * kv_append: the K and V rows of the k + 1 new tokens of every branch are written at the tail of
 * the branch's private cache, positions priv_len[b] - (k + 1) .. priv_len[b] - 1 (Section 2: the
 * drafted tokens are verified in one parallel forward, so their keys and values are in the cache
 * that forward's attention reads).  Dense layouts: Knew, Vnew [B][k+1][Hkv][D];
 * Kpriv, Vpriv [B][Hkv][Lmax][D]; es = bytes per element.  Positions outside [0, Lmax) are skipped.
 * ------------------------------------------------------------------------------------------- */
int oracle_kv_append(int B, int k, int Hkv, int D, int Lmax, int es, const void *Knew, const void *Vnew, void *Kpriv,
                     void *Vpriv, const int32_t *priv_len)
{
    if (B < 1 || k < 0 || Hkv < 1 || D < 1 || Lmax < 1 || (es != 2 && es != 4)) return -2;
    if (!Knew || !Vnew || !Kpriv || !Vpriv || !priv_len) return -1;
    const int R = k + 1;
    const size_t row = (size_t)D * (size_t)es;
    for (int b = 0; b < B; ++b)
        for (int r = 0; r < R; ++r) {
            const int64_t t = (int64_t)priv_len[b] - R + r;
            if (t < 0 || t >= Lmax) continue;
            for (int h = 0; h < Hkv; ++h) {
                const size_t src = (((size_t)b * R + r) * Hkv + h) * row;
                const size_t dst = (((size_t)b * Hkv + h) * Lmax + (size_t)t) * row;
                memcpy((char *)Kpriv + dst, (const char *)Knew + src, row);
                memcpy((char *)Vpriv + dst, (const char *)Vnew + src, row);
            }
        }
    return 0;
}
