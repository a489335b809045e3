// spec_accept: lossless speculative-sampling acceptance for B branches (the rule of the works
// the paper cites for speculative decoding in Section 2 / Section 3.2).
//
// Two launches, both bound by streaming fp32 rows from HBM:
//   accept_scan_kernel  grid (chunks, B): every workgroup re-derives the branch's accepted
//       length n from the 2k gathered probabilities, then turns its chunk of the row to be
//       sampled (residual max(0, p_n - q_n), or p_k) into 2^-40 fixed-point weights and writes
//       the chunk's integer sum.  One read of the stop row(s) -- the only V-sized traffic.
//   accept_pick_kernel  grid (B): scans the chunk sums, locates the chunk and then the token
//       where the integer CDF crosses T = floor(m * Z / 2^24); re-reads that one chunk only.
// All sums are 64-bit integers, so the result is independent of reduction order and equals a
// sequential scan bit for bit.
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

}  // namespace lotts

extern "C" size_t spec_accept_workspace_bytes(int32_t B, int32_t k, int32_t V) {
    if (B < 1 || k < 0 || k > lotts::kAccMaxK || V < 1 || B > 65535) return 0;
    const lotts::AcceptPlan pl = lotts::plan_accept(V);
    return (size_t)2 * B * pl.nchunks * sizeof(unsigned long long);
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
