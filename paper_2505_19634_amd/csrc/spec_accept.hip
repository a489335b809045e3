// spec_accept: lossless speculative-sampling acceptance for B branches (the rule of the works
// the paper cites for speculative decoding in Section 2 / Section 3.2).
//
// One launch when the vocabulary fits (accept_fused_kernel), two otherwise:
//   accept_fused_kernel  grid (S slices x B branches), 4 wavefronts per workgroup.  Every workgroup
//       re-derives the branch's accepted length n from the 2k gathered probabilities; each of its
//       wavefronts turns one sub-chunk of the row to be sampled (residual max(0, p_n - q_n), or p_k)
//       into 2^-40 fixed-point weights -- all of the sub-chunk's loads are requested before the first
//       is used -- and publishes the sub-chunk's integer sum as two 8-byte words, each carrying half
//       of it and this call's 32-bit tag.  The workgroup of a branch's LAST
//       slice then collects the branch's sums (it only ever waits for workgroups with smaller
//       block indices, which were dispatched before it; the wait is bounded), locates the sub-chunk
//       and the token where the integer CDF crosses T = floor(m * Z / 2^24), re-reading that one
//       sub-chunk only, and clears the published words.  An empty residual (possible only after a
//       draft of probability zero under both models) is resolved by that workgroup alone over the
//       row p_n.  One read of the stop row(s) -- the only
//       V-sized traffic -- and one launch: at these sizes the pass is bound by launch and memory
//       latency, not by bandwidth.
//   accept_scan_kernel + accept_pick_kernel  (V not a multiple of 4, unaligned rows, V > 2^18):
//       grid (chunks, B) writes chunk sums; a second launch (B) picks.
// All sums are 64-bit integers, so the result is independent of reduction order and equals a
// sequential scan bit for bit.
// Every floating-point operation in this file is rounded on its own, as the definition of the integer weights
// says: the compiler's default for device code would otherwise be free to merge a multiplication and a
// following addition or subtraction into one fused operation (one rounding), depending on how the
// surrounding code happens to be shaped.  Fused multiply-adds are written out where the definition has them.
#pragma clang fp contract(off)
#include "lotts_common.h"

namespace lotts {

constexpr int kAccThreads = 256;
constexpr int kAccWaves = kAccThreads / kWave;
constexpr int kAccMaxChunks = 1024;
constexpr int kAccMaxK = kAccThreads;  // one thread tests one draft position

struct AcceptPlan {
    int chunk;    // elements per chunk, a multiple of 4 * kAccThreads
    int nchunks;  // <= kAccMaxChunks
};

// 2048-token chunks (8 tokens per thread) unless the vocabulary needs more than kAccMaxChunks of them.
static inline AcceptPlan plan_accept(int V) {
    AcceptPlan pl;
    pl.chunk = 2048;
    while ((V + pl.chunk - 1) / pl.chunk > kAccMaxChunks) pl.chunk *= 2;
    pl.nchunks = (V + pl.chunk - 1) / pl.chunk;
    return pl;
}

// trunc(r * 2^40): the scaling is exact in fp32 and r <= 1, so the product is below 2^41.
__device__ __forceinline__ unsigned long long fixed_weight(float r) {
    return __float2ull_rz(r * 1099511627776.0f);
}
__device__ __forceinline__ float residual(float pv, float qv) {
    const float r = pv - qv;
    return r > 0.0f ? r : 0.0f;
}

// Number of drafts accepted before the first rejection; every thread of the block gets it.
__device__ __forceinline__ int accepted_length(int b, int k, int V, const float* __restrict__ p,
                                               const float* __restrict__ q, const int32_t* __restrict__ draft,
                                               const float* __restrict__ u, int* sh_first /*[kAccWaves]*/) {
    const int tid = threadIdx.x;
    bool rejected = false;
    if (tid < k) {
        int x = draft[(size_t)b * k + tid];
        x = x < 0 ? 0 : (x >= V ? V - 1 : x);
        const double pv = (double)p[((size_t)b * (k + 1) + tid) * V + x];
        const double qv = (double)q[((size_t)b * k + tid) * V + x];
        const double uv = (double)u[(size_t)b * (k + 1) + tid];
        rejected = !(uv * qv < pv);  // fp32 x fp32 is exact in fp64: the exact test u < p/q
    }
    const unsigned long long mask = __ballot(rejected);
    if ((tid & (kWave - 1)) == 0) sh_first[tid / kWave] = mask ? (tid + __ffsll((long long)mask) - 1) : k;
    __syncthreads();
    int n = k;
#pragma unroll
    for (int w = 0; w < kAccWaves; ++w) n = sh_first[w] < n ? sh_first[w] : n;
    return n;
}

// Block-wide sum of a pair of u64; result valid in every thread.
__device__ __forceinline__ void block_sum2(unsigned long long& a, unsigned long long& b,
                                           unsigned long long (*sh)[2] /*[kAccWaves][2]*/) {
    a = wave_sum_u64(a);
    b = wave_sum_u64(b);
    const int tid = threadIdx.x;
    __syncthreads();
    if ((tid & (kWave - 1)) == 0) {
        sh[tid / kWave][0] = a;
        sh[tid / kWave][1] = b;
    }
    __syncthreads();
    a = 0;
    b = 0;
#pragma unroll
    for (int w = 0; w < kAccWaves; ++w) {
        a += sh[w][0];
        b += sh[w][1];
    }
}

// Block-wide exclusive prefix sum of one u64 per thread (thread order); also returns nothing
// else: the caller already knows the total.
__device__ __forceinline__ unsigned long long block_excl_scan(unsigned long long v, unsigned long long* sh /*[kAccWaves]*/) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
    const unsigned long long incl = wave_incl_scan_u64(v, lane);
    __syncthreads();
    if (lane == kWave - 1) sh[w] = incl;
    __syncthreads();
    unsigned long long base = 0;
#pragma unroll
    for (int i = 0; i < kAccWaves; ++i) base += (i < w) ? sh[i] : 0ull;
    return base + incl - v;
}

template <bool VEC>
__global__ __launch_bounds__(kAccThreads) void accept_scan_kernel(int B, int k, int V, int chunk, int nchunks,
                                                                  const float* __restrict__ p,
                                                                  const float* __restrict__ q,
                                                                  const int32_t* __restrict__ draft,
                                                                  const float* __restrict__ u,
                                                                  int32_t* __restrict__ accept_len,
                                                                  unsigned long long* __restrict__ sums) {
    __shared__ int sh_first[kAccWaves];
    __shared__ unsigned long long sh_sum[kAccWaves][2];
    const int b = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
    const int n = accepted_length(b, k, V, p, q, draft, u, sh_first);
    if (c == 0 && tid == 0) accept_len[b] = n;

    const float* prow = p + ((size_t)b * (k + 1) + n) * V;
    const bool has_q = n < k;
    const float* qrow = has_q ? q + ((size_t)b * k + n) * V : prow;
    const int lo = c * chunk;
    const int hi = (lo + chunk < V) ? lo + chunk : V;
    unsigned long long s_res = 0, s_p = 0;
    if (VEC) {
        // two groups of 4 per row in flight: all four loads are issued before the first is used
        for (int i = lo + tid * 4; i < hi; i += kAccThreads * 8) {
            const int i2 = i + kAccThreads * 4;
            const bool in2 = i2 < hi;
            const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
            float4 pv[2] = {*reinterpret_cast<const float4*>(prow + i), zero};
            float4 qv[2] = {zero, zero};
            if (in2) pv[1] = *reinterpret_cast<const float4*>(prow + i2);
            if (has_q) {
                qv[0] = *reinterpret_cast<const float4*>(qrow + i);
                if (in2) qv[1] = *reinterpret_cast<const float4*>(qrow + i2);
            }
#pragma unroll
            for (int e = 0; e < 2; ++e) {  // zeros weigh nothing
                s_p += fixed_weight(pv[e].x) + fixed_weight(pv[e].y) + fixed_weight(pv[e].z) + fixed_weight(pv[e].w);
                s_res += fixed_weight(residual(pv[e].x, qv[e].x)) + fixed_weight(residual(pv[e].y, qv[e].y)) +
                         fixed_weight(residual(pv[e].z, qv[e].z)) + fixed_weight(residual(pv[e].w, qv[e].w));
            }
        }
    } else {
        for (int i = lo + tid; i < hi; i += kAccThreads) {
            const float pv = prow[i];
            const float qv = has_q ? qrow[i] : 0.f;
            s_p += fixed_weight(pv);
            s_res += fixed_weight(residual(pv, qv));
        }
    }
    block_sum2(s_res, s_p, sh_sum);
    if (tid == 0) {
        sums[(size_t)b * nchunks + c] = s_res;
        sums[(size_t)(B + b) * nchunks + c] = s_p;
    }
}

__global__ __launch_bounds__(kAccThreads) void accept_pick_kernel(int B, int k, int V, int chunk, int nchunks, bool vec,
                                                                  const float* __restrict__ p,
                                                                  const float* __restrict__ q,
                                                                  const float* __restrict__ u,
                                                                  const int32_t* __restrict__ accept_len,
                                                                  const unsigned long long* __restrict__ sums,
                                                                  int32_t* __restrict__ next_token) {
    __shared__ unsigned long long sh_sum[kAccWaves][2];
    __shared__ unsigned long long sh_scan[kAccWaves];
    __shared__ unsigned long long sh_base;
    __shared__ int sh_chunk;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int n = accept_len[b];

    // totals of both candidate rows: residual weights and plain p weights
    const int cpt = (nchunks + kAccThreads - 1) / kAccThreads;  // consecutive chunks per thread
    const int c0 = tid * cpt;
    unsigned long long t_res = 0, t_p = 0;
    for (int c = c0; c < c0 + cpt && c < nchunks; ++c) {
        t_res += sums[(size_t)b * nchunks + c];
        t_p += sums[(size_t)(B + b) * nchunks + c];
    }
    unsigned long long z_res = t_res, z_p = t_p;
    block_sum2(z_res, z_p, sh_sum);
    const bool use_res = (n < k) && (z_res != 0);  // an empty residual falls back to the row p_n
    const unsigned long long Z = use_res ? z_res : z_p;
    if (Z == 0) {
        if (tid == 0) next_token[b] = -1;
        return;
    }
    unsigned m = (unsigned)(u[(size_t)b * (k + 1) + k] * 16777216.0f);  // trunc(u * 2^24)
    m = m > 16777215u ? 16777215u : m;                                  // u must be < 1; keep T < Z regardless
    const unsigned long long T = (__umul64hi((unsigned long long)m, Z) << 40) | (((unsigned long long)m * Z) >> 24);

    // which chunk holds the crossing
    const unsigned long long* row_sums = sums + (size_t)(use_res ? b : B + b) * nchunks;
    const unsigned long long mine = use_res ? t_res : t_p;
    unsigned long long excl = block_excl_scan(mine, sh_scan);
    if (excl <= T && T < excl + mine) {  // exactly one thread: T < Z
        int c = c0;
        for (; c < c0 + cpt - 1 && c < nchunks - 1; ++c) {
            const unsigned long long s = row_sums[c];
            if (T < excl + s) break;
            excl += s;
        }
        sh_chunk = c;
        sh_base = excl;
    }
    __syncthreads();
    const int c = sh_chunk;
    const unsigned long long base = sh_base;

    // inside the chunk: thread t owns `ept` consecutive tokens
    const float* prow = p + ((size_t)b * (k + 1) + n) * V;
    const float* qrow = use_res ? q + ((size_t)b * k + n) * V : nullptr;
    const int ept = chunk / kAccThreads;
    const int lo = c * chunk + tid * ept;
    const int hi = (lo + ept < V) ? lo + ept : V;
    if (vec && ept == 8 && (c + 1) * chunk <= V) {  // uniform over the workgroup: both paths hold barriers
        // common case (a full chunk): the 8 weights stay in registers between the scan and the walk
        const float4 p0 = *reinterpret_cast<const float4*>(prow + lo), p1 = *reinterpret_cast<const float4*>(prow + lo + 4);
        float4 q0 = make_float4(0.f, 0.f, 0.f, 0.f), q1 = q0;
        if (use_res) {
            q0 = *reinterpret_cast<const float4*>(qrow + lo);
            q1 = *reinterpret_cast<const float4*>(qrow + lo + 4);
        }
        const float pv[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
        const float qv[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
        unsigned long long w[8], local = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            w[i] = fixed_weight(use_res ? residual(pv[i], qv[i]) : pv[i]);
            local += w[i];
        }
        unsigned long long run = base + block_excl_scan(local, sh_scan);
        if (run <= T && T < run + local) {
            int tok = lo;
#pragma unroll
            for (int i = 7; i >= 0; --i) {  // the first i whose inclusive prefix exceeds T
                unsigned long long pre = run;
#pragma unroll
                for (int j = 0; j <= i; ++j) pre += w[j];
                if (pre > T) tok = lo + i;
            }
            next_token[b] = tok;
        }
        return;
    }
    unsigned long long local = 0;
    for (int i = lo; i < hi; ++i) local += fixed_weight(use_res ? residual(prow[i], qrow[i]) : prow[i]);
    unsigned long long run = base + block_excl_scan(local, sh_scan);
    if (run <= T && T < run + local) {
        int tok = lo;
        for (int i = lo; i < hi; ++i) {
            run += fixed_weight(use_res ? residual(prow[i], qrow[i]) : prow[i]);
            if (run > T) {
                tok = i;
                break;
            }
        }
        next_token[b] = tok;
    }
}

// ---------------------------------------------------------------------------------------------
// single-launch path
// ---------------------------------------------------------------------------------------------
constexpr int kFuMaxSub = 64;        // sub-chunks per branch (one wavefront each): one wavefront scans their sums
constexpr int kFuMaxIter = 16;       // 16-byte loads per row and lane: sub-chunks of at most 4096 tokens
constexpr int kFuMaxV = kFuMaxSub * kFuMaxIter * 256;
constexpr int kFuSpinLimit = 1 << 18;  // polls of the collecting workgroup before it gives up (far beyond any real wait)

struct FusedPlan {
    int wlen;    // tokens per sub-chunk, a multiple of 256
    int iters;   // wlen / 256: 16-byte loads per row and lane, and tokens per thread in the pick
    int nsub;    // sub-chunks that hold tokens, <= kFuMaxSub
    int S;       // workgroups (slices of 4 sub-chunks) per branch
};
static inline FusedPlan plan_fused(int V) {
    FusedPlan pl;
    pl.wlen = ((V + kFuMaxSub - 1) / kFuMaxSub + 255) / 256 * 256;
    pl.iters = pl.wlen / 256;
    pl.nsub = (V + pl.wlen - 1) / pl.wlen;
    pl.S = (pl.nsub + kAccWaves - 1) / kAccWaves;
    return pl;
}

// trunc(r * 2^40) for 0 <= r <= 1 as two 32-bit conversions: hi = floor(r * 2^16), lo = floor(frac(r * 2^16) * 2^24);
// every step is exact (power-of-two scalings, fract), and hi * 2^24 + lo is the same integer as fixed_weight(r).
__device__ __forceinline__ void fixed_weight_split(float r, unsigned& hi, unsigned& lo) {
    const float a = fmaxf(r, 0.0f) * 65536.0f;  // negative and NaN inputs weigh nothing, as in fixed_weight
    hi = (unsigned)a;
    lo = (unsigned)(__builtin_amdgcn_fractf(a) * 16777216.0f);
}

// Sum over the wavefront of hi * 2^24 + lo with hi < 2^26 and lo < 2^30 per lane: the carry of lo moves into hi first, then
// both halves are summed as 32-bit values in two independent shuffle chains.  The total is valid in lane 0.
__device__ __forceinline__ unsigned long long wave_sum_split(unsigned hi, unsigned lo) {
    hi += lo >> 24;
    lo &= 0xffffffu;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        hi += __shfl_down(hi, d, kWave);
        lo += __shfl_down(lo, d, kWave);
    }
    return ((unsigned long long)hi << 24) + lo;
}
// Inclusive prefix sum over the wavefront of values below 2^58, as three limbs of 24 bits in independent 32-bit chains
// (a 64-bit shuffle chain costs twice the dependent steps).
__device__ __forceinline__ unsigned long long wave_incl_scan_limbs(unsigned long long v, int lane) {
    unsigned l0 = (unsigned)v & 0xffffffu, l1 = (unsigned)(v >> 24) & 0xffffffu, l2 = (unsigned)(v >> 48);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const unsigned o0 = __shfl_up(l0, d, kWave), o1 = __shfl_up(l1, d, kWave), o2 = __shfl_up(l2, d, kWave);
        if (lane >= d) {
            l0 += o0;
            l1 += o1;
            l2 += o2;
        }
    }
    return (unsigned long long)l0 + ((unsigned long long)l1 << 24) + ((unsigned long long)l2 << 48);
}

// one published word: half of a 64-bit sum under the call's tag
__device__ __forceinline__ unsigned long long tagged(unsigned half, unsigned tag) {
    return ((unsigned long long)tag << 32) | half;
}
__device__ __forceinline__ void publish(unsigned long long* slot, unsigned long long v) {
    __hip_atomic_store(slot, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long peek(const unsigned long long* slot) {
    return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The row a branch samples when its residual has no mass at all (only possible when a draft of probability zero under
// both models was "rejected", or for rows that are not distributions): the row p_n itself, handled by the collecting
// workgroup alone.  Thread t owns the tokens [t * E, (t + 1) * E); slow, and never on the path of a real workload.
__device__ __noinline__ int pick_plain_row(const float* __restrict__ prow, int V, unsigned m, unsigned long long* sh_scan) {
    const int tid = threadIdx.x;
    const int E = (V + kAccThreads - 1) / kAccThreads;
    const int lo = tid * E, hi = min(V, lo + E);
    unsigned long long local = 0;
    for (int i = lo; i < hi; ++i) local += fixed_weight(prow[i]);
    __shared__ unsigned long long sh_total;
    const unsigned long long excl = block_excl_scan(local, sh_scan);
    if (tid == kAccThreads - 1) sh_total = excl + local;
    __syncthreads();
    const unsigned long long Z = sh_total;
    if (Z == 0) return -1;
    const unsigned long long T = (__umul64hi((unsigned long long)m, Z) << 40) | (((unsigned long long)m * Z) >> 24);
    __shared__ int sh_tok;
    if (excl <= T && T < excl + local) {  // exactly one thread
        unsigned long long run = excl;
        int tok = lo;
        for (int i = lo; i < hi; ++i) {
            run += fixed_weight(prow[i]);
            if (run > T) {
                tok = i;
                break;
            }
        }
        sh_tok = tok;
    }
    __syncthreads();
    return sh_tok;
}

template <int MAXIT>
__global__ __launch_bounds__(kAccThreads) void accept_fused_kernel(int B, int k, int V, FusedPlan pl, unsigned tag,
                                                                   const float* __restrict__ p,
                                                                   const float* __restrict__ q,
                                                                   const int32_t* __restrict__ draft,
                                                                   const float* __restrict__ u,
                                                                   int32_t* __restrict__ accept_len,
                                                                   int32_t* __restrict__ next_token,
                                                                   unsigned long long* __restrict__ slots) {
    __shared__ int sh_first[kAccWaves];
    __shared__ unsigned long long sh_scan[kAccWaves];
    __shared__ unsigned long long sh_base, sh_T;
    __shared__ int sh_chunk, sh_bad;
    const int b = blockIdx.x / pl.S, s = blockIdx.x - b * pl.S;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid & (kWave - 1);
    const int n = accepted_length(b, k, V, p, q, draft, u, sh_first);

    // the row to sample: weights max(0, p_n - q_n) after a rejection, p_k when every draft was accepted
    const float* prow = p + ((size_t)b * (k + 1) + n) * V;
    const bool has_q = n < k;
    const float* qrow = has_q ? q + ((size_t)b * k + n) * V : prow;
    const int sub = s * kAccWaves + wave;          // this wavefront's sub-chunk of the row
    const int lo = sub * pl.wlen;
    // all of the sub-chunk is requested before any of it is used
    float4 pv[MAXIT], qv[MAXIT];
#pragma unroll
    for (int i = 0; i < MAXIT; ++i) {
        const int idx = lo + (i * kWave + lane) * 4;
        const bool in = i < pl.iters && idx < V;   // V is a multiple of 4 here: a group is inside or outside as a whole
        pv[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        qv[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (in) pv[i] = *reinterpret_cast<const float4*>(prow + idx);
        if (in && has_q) qv[i] = *reinterpret_cast<const float4*>(qrow + idx);
    }
    // per lane: at most 64 weights; their high parts (<= 2^16) and low parts (< 2^24) add up in 32 bits
    unsigned w_hi = 0, w_lo = 0;
#pragma unroll
    for (int i = 0; i < MAXIT; ++i) {
        const float pe[4] = {pv[i].x, pv[i].y, pv[i].z, pv[i].w};
        const float qe[4] = {qv[i].x, qv[i].y, qv[i].z, qv[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            unsigned h, l;
            fixed_weight_split(has_q ? residual(pe[e], qe[e]) : pe[e], h, l);
            w_hi += h;
            w_lo += l;
        }
    }
    const unsigned long long s_sub = wave_sum_split(w_hi, w_lo);
    unsigned long long* mine = slots + ((size_t)b * kFuMaxSub + sub) * 2;
    if (lane == 0 && sub < pl.nsub) {
        publish(mine + 0, tagged((unsigned)s_sub, tag));
        publish(mine + 1, tagged((unsigned)(s_sub >> 32), tag));
    }
    if (s != pl.S - 1) return;  // uniform over the workgroup

    // ---- the branch's last slice collects: it waits only for workgroups dispatched before it ----
    if (tid == 0) {
        accept_len[b] = n;
        sh_bad = 0;
    }
    __syncthreads();
    unsigned m = (unsigned)(u[(size_t)b * (k + 1) + k] * 16777216.0f);  // trunc(u * 2^24)
    m = m > 16777215u ? 16777215u : m;                                  // u must be < 1; keep T < Z regardless
    if (wave == 0) {
        unsigned long long v = 0;
        if (lane < pl.nsub) {
            unsigned long long* e = slots + ((size_t)b * kFuMaxSub + lane) * 2;
            unsigned long long w0 = 0, w1 = 0;
            bool ok = false;
            for (int spin = 0; spin < kFuSpinLimit; ++spin) {
                w0 = peek(e + 0);
                w1 = peek(e + 1);
                ok = (unsigned)(w0 >> 32) == tag && (unsigned)(w1 >> 32) == tag;
                if (ok) break;
                __builtin_amdgcn_s_sleep(1);
            }
            if (!ok) sh_bad = 1;  // never seen in practice: the producers were dispatched first and wait for nothing
            v = ((w1 & 0xffffffffull) << 32) | (w0 & 0xffffffffull);
            // the words are consumed: clear them, so that a captured launch (same tag) can be replayed
            publish(e + 0, 0ull);
            publish(e + 1, 0ull);
        }
        const unsigned long long incl = wave_incl_scan_limbs(v, lane);
        const unsigned long long Z = shfl_u64(incl, kWave - 1);
        const unsigned long long T = (__umul64hi((unsigned long long)m, Z) << 40) | (((unsigned long long)m * Z) >> 24);
        if (lane == 0) {
            sh_chunk = Z == 0 ? -1 : -2;  // -1: no mass in these weights; -2 is replaced by the lane that holds the crossing
            sh_T = T;
        }
        if (Z != 0 && incl - v <= T && T < incl) {  // exactly one lane: T < Z
            sh_chunk = lane;                        // after lane 0's store in the wavefront's program order
            sh_base = incl - v;
        }
    }
    __syncthreads();
    int c = sh_chunk;
    if (sh_bad) c = -3;
    if (c == -1 && has_q) {  // empty residual: the row p_n itself is sampled (uniform over the workgroup)
        const int tok = pick_plain_row(prow, V, m, sh_scan);
        if (tid == 0) next_token[b] = tok;
        return;
    }
    if (c < 0) {
        if (tid == 0) next_token[b] = -1;
        return;
    }
    const unsigned long long base = sh_base, T = sh_T;

    // inside the sub-chunk: thread t owns pl.iters consecutive tokens (served by the caches: just streamed)
    const int lo2 = c * pl.wlen + tid * pl.iters;
    float pw[MAXIT], qw[MAXIT];
#pragma unroll
    for (int i = 0; i < MAXIT; ++i) {
        const bool in = i < pl.iters && lo2 + i < V;
        pw[i] = in ? prow[lo2 + i] : 0.f;
        qw[i] = (in && has_q) ? qrow[lo2 + i] : 0.f;
    }
    unsigned long long w[MAXIT], local = 0;
#pragma unroll
    for (int i = 0; i < MAXIT; ++i) {
        unsigned h, l;
        fixed_weight_split(has_q ? residual(pw[i], qw[i]) : pw[i], h, l);
        w[i] = ((unsigned long long)h << 24) + l;
        local += w[i];
    }
    // exclusive prefix over the workgroup in thread order
    const unsigned long long incl = wave_incl_scan_limbs(local, lane);
    if (lane == kWave - 1) sh_scan[wave] = incl;
    __syncthreads();
    unsigned long long run = base + incl - local;
#pragma unroll
    for (int i = 0; i < kAccWaves; ++i) run += (i < wave) ? sh_scan[i] : 0ull;
    if (run <= T && T < run + local) {
        int tok = lo2;
        unsigned long long pre = run;
        bool found = false;
#pragma unroll
        for (int i = 0; i < MAXIT; ++i) {  // the first i whose inclusive prefix exceeds T
            pre += w[i];
            if (!found && pre > T) {
                tok = lo2 + i;
                found = true;
            }
        }
        next_token[b] = tok;
    }
}


}  // namespace lotts

extern "C" size_t spec_accept_workspace_bytes(int32_t B, int32_t k, int32_t V) {
    if (B < 1 || k < 0 || k > lotts::kAccMaxK || V < 1 || B > 65535) return 0;
    const lotts::AcceptPlan pl = lotts::plan_accept(V);
    const size_t two_launch = (size_t)2 * B * pl.nchunks * sizeof(unsigned long long);
    const size_t one_launch = (size_t)B * lotts::kFuMaxSub * 2 * sizeof(unsigned long long);
    return two_launch > one_launch ? two_launch : one_launch;  // the call picks the path from V and the pointers
}

extern "C" int spec_accept(int32_t B, int32_t k, int32_t V, const float* p, const float* q, const int32_t* draft,
                           const float* u, int32_t* accept_len, int32_t* next_token, void* workspace,
                           size_t workspace_bytes, void* stream) {
    using namespace lotts;
    if (B < 1 || k < 0 || k > kAccMaxK || V < 1 || B > 65535) return LOTTS_ERR_SHAPE;
    if (!p || !u || !accept_len || !next_token || !workspace) return LOTTS_ERR_NULL;
    if (k > 0 && (!q || !draft)) return LOTTS_ERR_NULL;
    if (workspace_bytes < spec_accept_workspace_bytes(B, k, V)) return LOTTS_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 7) != 0) return LOTTS_ERR_SHAPE;
    const AcceptPlan pl = plan_accept(V);
    unsigned long long* sums = static_cast<unsigned long long*>(workspace);
    hipStream_t s = (hipStream_t)stream;
    // float4 loads need every row start 16-byte aligned
    const bool vec = (V % 4 == 0) && (((uintptr_t)p & 15) == 0) && (k == 0 || ((uintptr_t)q & 15) == 0);
    if (vec && V <= kFuMaxV) {  // one launch
        const FusedPlan fp = plan_fused(V);
        const unsigned tag = next_word_tag();
        const dim3 fgrid((unsigned)((long long)B * fp.S));
        if (fp.iters <= 4)
            LOTTS_LAUNCH(accept_fused_kernel<4>, fgrid, dim3(kAccThreads), s, B, k, V, fp, tag, p, q, draft, u, accept_len,
                         next_token, sums);
        else if (fp.iters <= 8)
            LOTTS_LAUNCH(accept_fused_kernel<8>, fgrid, dim3(kAccThreads), s, B, k, V, fp, tag, p, q, draft, u, accept_len,
                         next_token, sums);
        else if (fp.iters <= 12)
            LOTTS_LAUNCH(accept_fused_kernel<12>, fgrid, dim3(kAccThreads), s, B, k, V, fp, tag, p, q, draft, u, accept_len,
                         next_token, sums);
        else
            LOTTS_LAUNCH(accept_fused_kernel<16>, fgrid, dim3(kAccThreads), s, B, k, V, fp, tag, p, q, draft, u, accept_len,
                         next_token, sums);
        return check_launch();
    }
    const dim3 grid(pl.nchunks, B);
    if (vec)
        LOTTS_LAUNCH(accept_scan_kernel<true>, grid, dim3(kAccThreads), s, B, k, V, pl.chunk, pl.nchunks, p,
                           q, draft, u, accept_len, sums);
    else
        LOTTS_LAUNCH(accept_scan_kernel<false>, grid, dim3(kAccThreads), s, B, k, V, pl.chunk, pl.nchunks, p,
                           q, draft, u, accept_len, sums);
    int rc = check_launch();
    if (rc != LOTTS_OK) return rc;
    LOTTS_LAUNCH(accept_pick_kernel, dim3(B), dim3(kAccThreads), s, B, k, V, pl.chunk, pl.nchunks, vec, p, q, u,
                       accept_len, sums, next_token);
    return check_launch();
}
