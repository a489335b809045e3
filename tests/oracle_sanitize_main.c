/* Drives every function of the CPU oracle over small random and edge-case inputs, with all buffers
 * allocated at their exact sizes, so that AddressSanitizer / UndefinedBehaviorSanitizer (the test
 * builds this file together with oracle/lotts_oracle.c under -fsanitize=address,undefined) see any
 * read or write out of bounds, any signed overflow or bad shift.  Test infrastructure only. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

int oracle_verify_attention(int B, int k, int Hq, int Hkv, int D, int P, int Lmax, int dtype, double scale, const void *Q,
                            const void *Kpre, const void *Vpre, const void *Kpriv, const void *Vpriv,
                            const int32_t *priv_len, double *O, double *lse);
int oracle_spec_accept(int B, int k, int V, const float *p, const float *q, const int32_t *draft, const float *u,
                       int32_t *accept_len, int32_t *next_token);
int oracle_majority_vote(int N, int B, const int32_t *answers, int32_t *winner, int32_t *winner_count);
uint64_t oracle_logit_weights(int V, const void *z, int dtype, float inv_temp, uint64_t *E);
int oracle_spec_accept_logits(int B, int k, int V, const void *zt, const void *zd, int dtype, float inv_temp,
                              const int32_t *draft, const float *u, int32_t *accept_len, int32_t *next_token,
                              int32_t *priv_len);
int oracle_confidence_vote(int N, int B, int T, const int32_t *answers, const float *conf, const int32_t *conf_len,
                           int weight_mode, int select_mode, int32_t *winner, float *winner_score);
int oracle_skinny_gemm(int M, int N, int K, int dtype, const void *X, const void *W, double *Y);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t next_u64(void)
{
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static double unif(void) { return (double)(next_u64() >> 11) / 9007199254740992.0; }
static float gauss(void) { return (float)(sqrt(-2.0 * log(unif() + 1e-300)) * cos(6.283185307179586 * unif())); }
static uint16_t to_bf16(float f)
{
    uint32_t b;
    memcpy(&b, &f, 4);
    return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}
/* n values ~ std * N(0,1), stored as fp32 (dtype 0) or bf16 (dtype 1), exactly n elements */
static void *normal_buf(size_t n, int dtype, float std)
{
    void *p = malloc((n ? n : 1) * (dtype ? 2 : 4));
    for (size_t i = 0; i < n; ++i) {
        float v = std * gauss();
        if (dtype)
            ((uint16_t *)p)[i] = to_bf16(v);
        else
            ((float *)p)[i] = v;
    }
    return p;
}
static float *softmax_rows(size_t rows, int V, float std)
{
    float *p = malloc(sizeof(float) * (rows * V ? rows * V : 1));
    for (size_t r = 0; r < rows; ++r) {
        double s = 0;
        for (int v = 0; v < V; ++v)
            s += (p[r * V + v] = expf(std * gauss()));
        for (int v = 0; v < V; ++v)
            p[r * V + v] = (float)(p[r * V + v] / s);
    }
    return p;
}
#define CHECK(x) do { if (!(x)) { fprintf(stderr, "check failed line %d: %s\n", __LINE__, #x); return 1; } } while (0)

static int attention_case(int B, int k, int Hq, int Hkv, int D, int P, int Lmax, int dtype, int ragged)
{
    const int R = k + 1;
    void *Q = normal_buf((size_t)B * R * Hq * D, dtype, 0.5f);
    void *Kp = normal_buf((size_t)Hkv * P * D, dtype, 0.5f), *Vp = normal_buf((size_t)Hkv * P * D, dtype, 0.5f);
    void *K = normal_buf((size_t)B * Hkv * Lmax * D, dtype, 0.5f), *V = normal_buf((size_t)B * Hkv * Lmax * D, dtype, 0.5f);
    int32_t *pl = malloc(sizeof(int32_t) * B);
    for (int b = 0; b < B; ++b)
        pl[b] = ragged ? R + (int)(next_u64() % (uint64_t)(Lmax - R + 1)) : Lmax;
    double *O = malloc(sizeof(double) * (size_t)B * R * Hq * D), *lse = malloc(sizeof(double) * (size_t)B * R * Hq);
    CHECK(oracle_verify_attention(B, k, Hq, Hkv, D, P, Lmax, dtype, ragged ? 0.2 : 0.0, Q, P ? Kp : NULL, P ? Vp : NULL, K,
                                  V, pl, O, lse) == 0);
    for (size_t i = 0; i < (size_t)B * R * Hq * D; ++i)
        CHECK(isfinite(O[i]));
    CHECK(oracle_verify_attention(B, k, Hq, Hkv, D, P, Lmax, dtype, 0.0, Q, Kp, Vp, K, V, pl, O, NULL) == 0);
    free(Q); free(Kp); free(Vp); free(K); free(V); free(pl); free(O); free(lse);
    return 0;
}

static int accept_case(int B, int k, int V)
{
    float *p = softmax_rows((size_t)B * (k + 1), V, 2.0f), *q = softmax_rows((size_t)B * k, V, 2.0f);
    int32_t *draft = malloc(sizeof(int32_t) * (B * k ? B * k : 1));
    float *u = malloc(sizeof(float) * B * (k + 1));
    for (int i = 0; i < B * k; ++i)
        draft[i] = (int32_t)(next_u64() % (uint64_t)V);
    for (int i = 0; i < B * (k + 1); ++i)
        u[i] = (float)(next_u64() >> 40) / 16777216.0f;
    if (B > 1 && k > 0) { /* degenerate rows: all mass on one token, an empty residual, a zero row */
        memset(p + (size_t)1 * (k + 1) * V, 0, sizeof(float) * V);
        memcpy(q, p, sizeof(float) * V);
    }
    int32_t *n = malloc(sizeof(int32_t) * B), *t = malloc(sizeof(int32_t) * B);
    CHECK(oracle_spec_accept(B, k, V, p, k ? q : NULL, k ? draft : NULL, u, n, t) == 0);
    for (int b = 0; b < B; ++b)
        CHECK(n[b] >= 0 && n[b] <= k && t[b] >= -1 && t[b] < V);
    free(p); free(q); free(draft); free(u); free(n); free(t);
    return 0;
}

static int logits_case(int B, int k, int V, int dtype, float inv_temp)
{
    void *zt = normal_buf((size_t)B * (k + 1) * V, dtype, 2.0f), *zd = normal_buf((size_t)B * k * V, dtype, 2.0f);
    if (!dtype && V > 2) { /* -inf logits and a huge spread */
        ((float *)zt)[1] = -INFINITY;
        ((float *)zt)[2] = 300.0f;
    }
    int32_t *draft = malloc(sizeof(int32_t) * (B * k ? B * k : 1));
    float *u = malloc(sizeof(float) * B * (k + 1));
    for (int i = 0; i < B * k; ++i)
        draft[i] = (int32_t)(next_u64() % (uint64_t)V);
    for (int i = 0; i < B * (k + 1); ++i)
        u[i] = (float)(next_u64() >> 40) / 16777216.0f;
    int32_t *n = malloc(sizeof(int32_t) * B), *t = malloc(sizeof(int32_t) * B), *pl = malloc(sizeof(int32_t) * B);
    for (int b = 0; b < B; ++b)
        pl[b] = 1000 + b;
    CHECK(oracle_spec_accept_logits(B, k, V, zt, k ? zd : NULL, dtype, inv_temp, k ? draft : NULL, u, n, t, pl) == 0);
    for (int b = 0; b < B; ++b)
        CHECK(n[b] >= 0 && n[b] <= k && t[b] >= 0 && t[b] < V && pl[b] == 1000 + b - (k - n[b]));
    uint64_t *E = malloc(sizeof(uint64_t) * V);
    CHECK(oracle_logit_weights(V, zt, dtype, inv_temp, E) > 0);
    free(zt); free(zd); free(draft); free(u); free(n); free(t); free(pl); free(E);
    return 0;
}

static int votes_case(int N, int B, int T)
{
    int32_t *a = malloc(sizeof(int32_t) * N * B), *cl = malloc(sizeof(int32_t) * N * B);
    float *c = malloc(sizeof(float) * (size_t)N * B * T);
    for (int i = 0; i < N * B; ++i) {
        a[i] = (int32_t)(next_u64() % 7) - 1;
        cl[i] = (int32_t)(next_u64() % (uint64_t)(T + 1));
    }
    for (size_t i = 0; i < (size_t)N * B * T; ++i)
        c[i] = (float)unif();
    int32_t *w = malloc(sizeof(int32_t) * N), *cnt = malloc(sizeof(int32_t) * N);
    float *sc = malloc(sizeof(float) * N);
    CHECK(oracle_majority_vote(N, B, a, w, cnt) == 0);
    for (int wm = 0; wm < 2; ++wm)
        for (int sm = 0; sm < 2; ++sm) {
            CHECK(oracle_confidence_vote(N, B, T, a, c, cl, wm, sm, w, sc) == 0);
            CHECK(oracle_confidence_vote(N, B, T, a, c, NULL, wm, sm, w, sc) == 0);
        }
    free(a); free(cl); free(c); free(w); free(cnt); free(sc);
    return 0;
}

static int gemm_case(int M, int N, int K, int dtype)
{
    void *X = normal_buf((size_t)M * K, dtype, 1.0f), *W = normal_buf((size_t)N * K, dtype, 0.1f);
    double *Y = malloc(sizeof(double) * (size_t)M * N);
    CHECK(oracle_skinny_gemm(M, N, K, dtype, X, W, Y) == 0);
    free(X); free(W); free(Y);
    return 0;
}

int main(void)
{
    int bad = 0;
    bad |= attention_case(2, 3, 4, 4, 64, 32, 64, 0, 0);   /* the tiny fp32 config */
    bad |= attention_case(3, 2, 8, 2, 16, 5, 11, 1, 1);    /* bf16, GQA, ragged lengths, explicit scale */
    bad |= attention_case(1, 0, 2, 1, 8, 0, 1, 0, 0);      /* k = 0, no prefix, a single key */
    bad |= attention_case(2, 4, 6, 3, 32, 7, 5, 1, 0);     /* private cache = the new tokens only */
    bad |= accept_case(5, 3, 37);
    bad |= accept_case(2, 0, 9);
    bad |= accept_case(3, 2, 1);
    bad |= logits_case(4, 3, 50, 0, 1.0f);
    bad |= logits_case(3, 2, 33, 1, 0.7f);
    bad |= logits_case(2, 0, 1, 0, 2.0f);
    bad |= votes_case(3, 17, 9);
    bad |= votes_case(1, 1, 1);
    bad |= gemm_case(5, 16, 128, 1);
    bad |= gemm_case(3, 7, 5, 0);
    /* argument errors return -1 without touching anything */
    bad |= oracle_verify_attention(0, 1, 4, 4, 8, 0, 4, 0, 0.0, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) != -1;
    bad |= oracle_spec_accept(1, 1, 0, NULL, NULL, NULL, NULL, NULL, NULL) != -1;
    bad |= oracle_majority_vote(1, 0, NULL, NULL, NULL) != -1;
    if (bad) {
        fprintf(stderr, "oracle sanitize driver: FAILED\n");
        return 1;
    }
    printf("oracle sanitize driver: ok\n");
    return 0;
}
