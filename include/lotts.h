/*
 * lotts.h -- C ABI of the MI355X (gfx950) speculative verification step run across B
 * concurrent reasoning branches: the hot path of latency-optimal test-time scaling
 * ("Faster and Better LLMs via Latency-Aware Test-Time Scaling", arXiv 2505.19634).
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees or synchronises; work is enqueued on `stream` (a hipStream_t passed
 *     as void*, NULL = the default stream) and outputs are fully overwritten.
 *   - Return value: LOTTS_OK or a negative lotts_status.  All argument checks run on the
 *     host before anything is launched; a failed call launches nothing.
 *   - Scratch memory is passed in as `workspace`; the *_workspace_bytes queries say how much.
 *     Calls that share a workspace must be ordered on one stream.  spec_accept and
 *     spec_accept_logits take any contents, each other's leftovers included (what their kernels
 *     exchange carries a tag that no other call of the process has).  A buffer given to
 *     verify_attention stays verify_attention's: it keeps arrival cells in the first 128 KiB,
 *     the buffer must be ZERO-FILLED ONCE before its first use (hipMemset or a fill kernel),
 *     and again if another entry point has written to it in between.
 *     After that it serves any number of calls of any geometry without clearing: every cell
 *     carries the tag of the call that wrote it (tags grow from call to call within the
 *     process), a call treats whatever an earlier call left there as zero arrivals, and a
 *     call that completes leaves its cells zero.  So a call that never completed (a failed
 *     launch, an aborted stream) does not spoil the buffer for the calls after it.  The one
 *     exception is a captured launch that is replayed later: it keeps the tag it was captured
 *     with, so clear the buffer before replaying a graph after some call on it was aborted.
 */
#ifndef LOTTS_H
#define LOTTS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LOTTS_OK = 0,
    LOTTS_ERR_NULL = -1,       /* a required pointer is NULL */
    LOTTS_ERR_SHAPE = -2,      /* sizes or strides the kernels cannot take */
    LOTTS_ERR_DTYPE = -3,      /* unknown element type */
    LOTTS_ERR_WORKSPACE = -4,  /* workspace smaller than *_workspace_bytes */
    LOTTS_ERR_LAUNCH = -5      /* the HIP runtime refused a launch */
} lotts_status;

typedef enum { LOTTS_F32 = 0, LOTTS_BF16 = 1 } lotts_dtype;

/* Human-readable text for a status code; never NULL. */
const char *lotts_strerror(int status);

/*
 * Geometry of one verify_attention call.
 * R = k + 1 query rows per branch: the k draft tokens (Section 3.3: draft length gamma) plus
 * the bonus position.  Query head h reads KV head h / (Hq / Hkv).
 * Strides are in ELEMENTS; the innermost D elements of every row are contiguous.
 * K and V of the same segment use the same strides.
 */
typedef struct {
    int32_t B;        /* concurrent branches (Section 3.2, branch-wise parallelism), >= 1; B * Hkv <= 16384 */
    int32_t k;        /* draft tokens per branch (sequence-wise parallelism), >= 0 */
    int32_t Hq, Hkv;  /* query / KV heads, Hq % Hkv == 0 */
    int32_t D;        /* head dimension: 64 or 128 */
    int32_t P;        /* tokens of the prompt prefix shared by all branches, >= 0 */
    int32_t Lmax;     /* allocated private tokens per branch, >= k + 1 */
    int32_t dtype;    /* lotts_dtype of Q, K, V and O */
    float scale;      /* softmax scale; 0 selects 1 / sqrt(D) */
    int64_t q_stride_b, q_stride_r, q_stride_h;              /* Q  [B][R][Hq][D] */
    int64_t kpre_stride_h, kpre_stride_t;                    /* Kpre, Vpre [Hkv][P][D] */
    int64_t kpriv_stride_b, kpriv_stride_h, kpriv_stride_t;  /* Kpriv, Vpriv [B][Hkv][Lmax][D] */
    int64_t o_stride_b, o_stride_r, o_stride_h;              /* O  [B][R][Hq][D] */
} lotts_attn_desc;

/* Bytes of workspace verify_attention needs for this geometry; 0 if the descriptor is invalid or the
 * partials of this geometry would not fit the 2 GiB that the kernels address with 32-bit offsets
 * (verify_attention then returns LOTTS_ERR_SHAPE). */
size_t verify_attention_workspace_bytes(const lotts_attn_desc *desc);

/*
 * verify_attention -- the target model's causal attention for the k + 1 new positions of
 * every branch (Section 2, speculative decoding: the target verifies the drafts in one
 * parallel forward; Section 3.1: the step is bound by loading the KV cache), one layer.
 *
 *   O[b][i][h][:] = sum_j softmax_j(scale * <Q[b][i][h], K_j>) * V_j
 * over the keys visible to row i of branch b: all P prefix keys, then the first
 * priv_len[b] - k + i private keys of branch b (the last k + 1 private positions are the new
 * tokens themselves; row i sees itself and the earlier ones).  The prefix K/V exist once and
 * are read from HBM once, whatever B is.
 *
 *   Q      [B][R][Hq][D]        dtype, strides from desc
 *   Kpre, Vpre   [Hkv][P][D]    dtype; may be NULL iff P == 0
 *   Kpriv, Vpriv [B][Hkv][Lmax][D] dtype
 *   priv_len [B] int32: private tokens of branch b INCLUDING its k + 1 new tokens.
 *            Contract k + 1 <= priv_len[b] <= Lmax.  It is device data and is not checked on
 *            the host: the kernels clamp it into that range, so nothing is read out of
 *            bounds, but the rows of an offending branch are then unspecified.
 *   O      [B][R][Hq][D] dtype, out
 *   lse    [B][R][Hq] fp32, out, may be NULL: natural-log sum of exp of the scaled scores
 *   workspace: >= verify_attention_workspace_bytes(desc), 16-byte aligned, zero-filled before first use
 *            (see above: arrival cells).  Calls that may overlap in time -- different streams --
 *            need workspaces of their own; calls on one stream can share one.
 * bf16 inputs are multiplied on the matrix cores with fp32 accumulation; fp32 inputs are
 * computed in fp32 throughout.
 */
int verify_attention(const lotts_attn_desc *desc, const void *Q, const void *Kpre, const void *Vpre,
                     const void *Kpriv, const void *Vpriv, const int32_t *priv_len, void *O, float *lse,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * verify_attention_noalloc -- verify_attention for callers that cannot allocate device memory or
 * hand over a workspace: code that runs under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same operation, same kernels, same results bit for bit; the arrival
 * cells and partials live in a 16 MiB scratch array built into the library (static device
 * memory: each GPU the library runs on holds its copy until the process ends) instead of a
 * caller's workspace.  The call allocates and frees nothing and calls no allocating routine.
 *   Limit: geometries with verify_attention_workspace_bytes(desc) > 16 MiB (16777216 bytes) are
 *   rejected with LOTTS_ERR_WORKSPACE before anything is launched; use verify_attention for those.
 *   The device that `stream` belongs to must be the calling thread's current device (the scratch
 *   address is looked up once per device, on the first call made there).
 *   All calls on one GPU share that GPU's scratch array, so calls that may overlap in time on one
 *   GPU (different streams, several host threads) race; order them on one stream.  Nothing has to
 *   be cleared between calls.
 * Arguments and errors otherwise as for verify_attention.
 */
int verify_attention_noalloc(const lotts_attn_desc *desc, const void *Q, const void *Kpre, const void *Vpre,
                             const void *Kpriv, const void *Vpriv, const int32_t *priv_len, void *O, float *lse,
                             void *stream);

/* Bytes of workspace spec_accept needs (0 if the sizes are invalid). */
size_t spec_accept_workspace_bytes(int32_t B, int32_t k, int32_t V);

/*
 * spec_accept -- lossless speculative-sampling acceptance per branch (the rule of the works
 * Section 2 cites for speculative decoding): draft token x_j is accepted iff
 * u_j < min(1, p_j(x_j) / q_j(x_j)), tested exactly as u_j * q_j(x_j) < p_j(x_j) in fp64;
 * accept_len[b] = n counts the drafts accepted before the first rejection.  The next token is
 * drawn from norm(max(0, p_n - q_n)) if n < k, from p_k otherwise, by inverting an integer
 * fixed-point CDF: w_v = trunc(r_v * 2^40), Z = sum_v w_v, T = floor(trunc(u[b][k] * 2^24) * Z
 * / 2^24), token = first v with w_0 + ... + w_v > T.  Integer sums make the result the same
 * for any reduction order.  If the residual has no mass the row p_n itself is sampled; if that
 * has none either, next_token = -1.
 *
 *   1 <= B <= 65535, 0 <= k <= 256, V >= 1
 *   p [B][k+1][V] fp32  target probabilities (finite, >= 0)
 *   q [B][k][V]   fp32  draft probabilities; NULL iff k == 0
 *   draft [B][k]  int32 draft tokens in [0, V) (the kernel clamps); NULL iff k == 0
 *   u [B][k+1]    fp32  uniforms in [0, 1)
 *   accept_len [B] int32 out, in [0, k];  next_token [B] int32 out, in [0, V) or -1
 *   workspace: >= spec_accept_workspace_bytes(B, k, V), 8-byte aligned, any contents (what the kernels
 *       exchange through it is validated by a tag that differs from call to call)
 * One launch when V is a multiple of 4, at most 2^18, and the rows are 16-byte aligned; two otherwise.
 */
int spec_accept(int32_t B, int32_t k, int32_t V, const float *p, const float *q, const int32_t *draft,
                const float *u, int32_t *accept_len, int32_t *next_token, void *workspace,
                size_t workspace_bytes, void *stream);

/* Bytes of workspace spec_accept_logits needs (0 if the sizes are invalid). */
size_t spec_accept_logits_workspace_bytes(int32_t B, int32_t k, int32_t V);

/*
 * spec_accept_logits -- the same acceptance rule as spec_accept, taken straight from the target
 * and draft LOGITS (Section 2: the draft model proposes, the target model verifies), so the
 * V-wide softmax outputs never go through memory.  The distributions are
 * softmax(z * inv_temperature), defined on integers so that the result does not depend on
 * summation order or on an exp() implementation:
 *   y_v = fp32(z_v) * inv_temperature, m = max_v y_v, t_v = (y_v - m) * log2(e)   (fp32, each
 *   operation rounded once), E_v = trunc(P(frac(-t_v)) * 2^(30 - floor(-t_v))), 0 when
 *   floor(-t_v) >= 31, where P(f) = 1 + f(c1 + f(c2 + ... + f c6)) evaluated by fused
 *   multiply-adds approximates 2^-f on [0, 1) to 1.4e-7 with (c1..c6) = (-0x1.62e430p-1,
 *   0x1.ebfbaap-3, -0x1.c6a66cp-5, 0x1.3a7ae4p-7, -0x1.52a284p-10, 0x1.e243bep-14);
 *   S = sum_v E_v; the probability of token v is E_v / S exactly.
 * Draft x_j is accepted iff U_j * Eq_j(x_j) * Sp_j < 2^24 * Ep_j(x_j) * Sq_j, U_j = trunc(u_j * 2^24)
 * (the test u < min(1, p/q) on these rationals).  After the first rejection at n the next token
 * is drawn with weights W_v = max(0, Ep_n(v) * Sq_n - Eq_n(v) * Sp_n) (the row Ep_n if all W are 0);
 * if all k drafts are accepted, with weights Ep_k(v).  token = first v with
 * W_0 + ... + W_v > floor(trunc(u[b][k] * 2^24) * sum(W) / 2^24).  All in 128-bit integers.
 *
 *   1 <= B <= 65535, 0 <= k <= 256, 1 <= V <= 2^20, ceil(V / 16384) * B * (2k + 1) < 2^31
 *   target_logits [B][k+1][V], draft_logits [B][k][V] (NULL iff k == 0): logit_dtype = LOTTS_F32 or
 *       LOTTS_BF16, finite or -inf; inv_temperature > 0.  A sampled row without any weight (every
 *       logit -inf) yields next_token = -1, as in spec_accept.
 *   draft [B][k] int32 (NULL iff k == 0), u [B][k+1] fp32 in [0, 1)
 *   accept_len [B], next_token [B] int32 out
 *   priv_len [B] int32 in/out, NULL to skip: the private length verify_attention was given for
 *       this step (it counts the k + 1 new tokens).  The k - accept_len[b] rejected drafts are
 *       dropped from it, priv_len[b] -= k - accept_len[b], so it then counts exactly the tokens
 *       whose keys and values stay valid; the caller appends the next step's k + 1 tokens there.
 *   workspace: >= spec_accept_logits_workspace_bytes(B, k, V), 16-byte aligned, any contents
 */
int spec_accept_logits(int32_t B, int32_t k, int32_t V, const void *target_logits, const void *draft_logits,
                       int32_t logit_dtype, float inv_temperature, const int32_t *draft, const float *u,
                       int32_t *accept_len, int32_t *next_token, int32_t *priv_len, void *workspace,
                       size_t workspace_bytes, void *stream);

/*
 * majority_vote -- the answer most branches agree on (Section 1 and Section 4.1: branches are
 * aggregated by majority voting), for N independent questions at once.
 *
 *   answers [N][B] int32: answer id of each branch; ids < 0 mean "no answer" and do not count
 *   winner [N], winner_count [N] int32 out: the id with the most votes and its votes; ties go
 *   to the id whose first occurrence has the smallest branch index; (-1, 0) if no branch
 *   answered.  1 <= B <= 4096.
 */
int majority_vote(int32_t N, int32_t B, const int32_t *answers, int32_t *winner, int32_t *winner_count,
                  void *stream);

/*
 * confidence_vote -- confidence-based aggregation of the branches' answers (Section "Different
 * Aggregation Strategies"): every branch's answer is weighted by the minimum or the average of
 * its confidence scores; then either the single most confident answer wins ("max"), or the
 * weights of identical answers are added and the largest total wins ("vote").
 *
 *   answers [N][B] int32 (id < 0: no answer), conf [N][B][T] fp32 in [0, 1],
 *   conf_len [N][B] int32 valid scores per branch (NULL: all T)
 *   weight_mode 0 = min, 1 = avg;  select_mode 0 = max, 1 = vote;  1 <= B <= 1024
 *   winner [N] int32, winner_score [N] fp32 out; (-1, 0) if no branch takes part
 * Scores are quantised to trunc(c * 2^30) so that sums are integers; a branch's weight is
 * q_min / 2^30 or sum(q) / (len * 2^30), formed in fp64 and rounded once to fp32; "vote" adds the
 * fp32 weights of identical answers in branch order; ties go to the earliest branch (max) or the
 * earliest first occurrence (vote).  Branches without an answer or without scores are left out.
 */
int confidence_vote(int32_t N, int32_t B, int32_t T, const int32_t *answers, const float *conf,
                    const int32_t *conf_len, int32_t weight_mode, int32_t select_mode, int32_t *winner,
                    float *winner_score, void *stream);

/*
 * kv_append -- put the K and V rows of the k + 1 new tokens of every branch at the tail of that
 * branch's private cache, where verify_attention expects them (Section 2: the target verifies the
 * drafted tokens in one parallel forward, so their keys and values join the cache before the
 * attention of that forward; together with the length roll-back of spec_accept_logits this is the
 * cache side of one speculative step).
 *   Kpriv[b][h][priv_len[b] - (k + 1) + r][:] = Knew[b][r][h][:]   for r = 0 .. k; V likewise
 *   Knew, Vnew: [B][k+1][Hkv][D] views (element strides new_stride_b / _r / _h, D contiguous), e.g. the K
 *       and V columns of a QKV projection's output; V uses the same strides as K
 *   Kpriv, Vpriv: [B][Hkv][Lmax][D] in/out (element strides priv_stride_b / _h / _t, as in lotts_attn_desc)
 *   priv_len [B] int32 (device): private tokens of branch b INCLUDING the k + 1 new ones; positions
 *       outside [0, Lmax) are skipped (a violated contract never writes out of bounds)
 *   dtype: LOTTS_BF16 or LOTTS_F32, of all four buffers; a row of D elements is a multiple of 16
 *       bytes, and all pointers and strides are 16-byte aligned
 * A plain copy: bit-exact; nothing else in the caches is touched.
 */
int kv_append(int32_t B, int32_t k, int32_t Hkv, int32_t D, lotts_dtype dtype, const void *Knew, const void *Vnew,
              int64_t new_stride_b, int64_t new_stride_r, int64_t new_stride_h, void *Kpriv, void *Vpriv,
              int64_t priv_stride_b, int64_t priv_stride_h, int64_t priv_stride_t, int32_t Lmax,
              const int32_t *priv_len, void *stream);

/* Bytes of workspace skinny_gemm needs (0 if the sizes are invalid). */
size_t skinny_gemm_workspace_bytes(int32_t M, int32_t N, int32_t K);

/*
 * skinny_gemm -- one weight GEMM of the verify forward: the B * (k + 1) new tokens against a
 * Linear layer's weight (Section 3.1: the step is bound by loading the weights; Appendix: 64 GB of
 * weights for the 32B model).
 *   Y[m][n] = sum_k X[m][k] * W[n][k]
 *   X [M][K] bf16 (row pitch ldx elements), W [N][K] bf16 (ldw), Y [M][N] bf16 out (ldy)
 *   1 <= M <= 256; N a multiple of 8; K a multiple of 128; ldx, ldw multiples of 8, ldy of 4;
 *   X, W, workspace 16-byte aligned, Y 8-byte aligned
 * bf16 products accumulate in fp32 on the matrix cores; W is read from HBM once.  When N is
 * small the K range is split over workgroups and the fp32 partials are summed in a fixed order
 * by a second launch (deterministic).
 *   workspace: >= skinny_gemm_workspace_bytes(M, N, K), any contents
 */
int skinny_gemm(int32_t M, int32_t N, int32_t K, const void *X, int64_t ldx, const void *W, int64_t ldw, void *Y,
                int64_t ldy, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Kernel timer -- device execution time of the kernels the entry points launch, for callers that
 * have no profiler at hand (not an operation of the paper; a measurement aid).
 * Between lotts_timer_start and lotts_timer_stop every kernel launched by the CALLING HOST THREAD
 * through this library carries a pair of events of its own, attached to the dispatch, which read
 * that kernel's start and end on the device; the gaps between commands are not included.
 *   lotts_timer_start(max_launches): 1 <= max_launches <= 2^20.  Launches beyond max_launches are
 *       not timed.  Creates the events it needs the first time (host allocation only).
 *   lotts_timer_pause(paused): nonzero = launches are not timed until lotts_timer_pause(0); host
 *       flag only, so single calls of a pipelined loop can be picked out without waiting for the
 *       device (a timed launch costs the host and the queue a few microseconds more than a plain one).
 *   lotts_timer_stop(launches, ms): waits for the timed kernels to finish, writes their number to
 *       *launches and, if ms is not NULL, each one's milliseconds to ms[0 .. *launches), in launch
 *       order (HOST array of at least max_launches floats).  Switches the timer off.
 * The order of launches inside one call: verify_attention 1 (2 when the partials of a row are
 * many: attention, then merge); spec_accept 1 (2 -- scan, pick -- when V is not a multiple of 4, beyond
 * 2^18, or the rows are not 16-byte aligned); spec_accept_logits 3 (max, sum,
 * scan and pick); majority_vote 1; confidence_vote 1; skinny_gemm 1 (2 when K is split: GEMM, reduce).
 */
int lotts_timer_start(int32_t max_launches);
int lotts_timer_pause(int32_t paused);
int lotts_timer_stop(int32_t *launches, float *ms);

/*
 * greedy_search -- the search for the latency-optimal configuration (B*, gamma*) of Algorithm 1
 * (Section 3.3).  HOST function: it launches nothing; `tts_task(B, gamma, T, user)` is the
 * caller's evaluation of the accuracy reached with B branches and draft length gamma under the
 * latency budget T.  From (1, 0), each round evaluates (2B, gamma) and (B, gamma + 1), moves to
 * the better one (the branch move on a tie) if it is strictly better than the current accuracy,
 * and stops otherwise.  Moves beyond B_max / gamma_max are not evaluated.
 *   B_opt, gamma_opt, acc_opt: out, required.  rounds (iterations of the loop, the terminating
 *   one included: log2 B* + gamma* + 1 when no bound binds) and evaluations (calls of tts_task):
 *   out, may be NULL.
 */
typedef double (*lotts_tts_task_fn)(int32_t B, int32_t gamma, double T, void *user);
int greedy_search(lotts_tts_task_fn tts_task, void *user, double T, int32_t B_max, int32_t gamma_max,
                  int32_t *B_opt, int32_t *gamma_opt, double *acc_opt, int32_t *rounds, int32_t *evaluations);

#ifdef __cplusplus
}
#endif
#endif /* LOTTS_H */
