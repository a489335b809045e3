// confidence_vote: confidence-based aggregation of the branches' answers (paper Section
// "Different Aggregation Strategies"): weight each answer by the min / avg of the branch's
// confidence scores, then pick the most confident answer ("max") or add up the weights of
// identical answers ("vote").  One workgroup per question: the B rows of T scores are reduced
// one after the other by all 256 threads (integer sums, so the order inside a row does not
// matter), the selection runs over the B weights in LDS.  Latency-bound, like majority_vote.
// Every floating-point operation in this file is rounded on its own, as the definition of the integer weights
// says: the compiler's default for device code would otherwise be free to merge a multiplication and a
// following addition or subtraction into one fused operation (one rounding), depending on how the
// surrounding code happens to be shaped.  Fused multiply-adds are written out where the definition has them.
#pragma clang fp contract(off)
#include "lotts_common.h"

namespace lotts {

constexpr int kConfThreads = 256;
constexpr int kConfMaxB = 1024;

__global__ __launch_bounds__(kConfThreads) void confidence_vote_kernel(int B, int T, const int32_t* __restrict__ answers,
                                                                       const float* __restrict__ conf,
                                                                       const int32_t* __restrict__ conf_len,
                                                                       int weight_mode, int select_mode,
                                                                       int32_t* __restrict__ winner,
                                                                       float* __restrict__ winner_score) {
    __shared__ int32_t a[kConfMaxB];
    __shared__ float w[kConfMaxB];
    __shared__ unsigned long long sh_key[kConfThreads / kWave];
    const int n = blockIdx.x, tid = threadIdx.x;
    // weights: groups of LPB lanes (a power of two, at most one wavefront) reduce one branch's scores
    // with shuffles; 256 / LPB branches are in flight at a time.  a[b] = -1 marks a branch left out.
    int LPB = kWave;
    while (LPB > 1 && (kConfThreads / LPB) < B) LPB >>= 1;
    const int per_pass = kConfThreads / LPB;
    const int sub = tid & (LPB - 1);
    for (int b0 = 0; b0 < B; b0 += per_pass) {
        const int b = b0 + tid / LPB;
        const bool in = b < B;
        int ans = -1, len = 0;
        if (in) {
            ans = answers[(size_t)n * B + b];
            len = conf_len ? conf_len[(size_t)n * B + b] : T;
            len = len > T ? T : len;
        }
        unsigned long long sum = 0, mn = ~0ull;
        if (in && ans >= 0) {
            const float* c = conf + ((size_t)n * B + b) * T;
            // 16 independent loads at a time: one load per iteration would cost a memory latency each
            for (int t0 = sub; t0 < len; t0 += 16 * LPB) {
                float v[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int t = t0 + e * LPB;
                    v[e] = c[t < len ? t : len - 1];
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const unsigned long long q = __float2ull_rz(v[e] * 1073741824.0f);  // trunc(c * 2^30)
                    const bool use = t0 + e * LPB < len;
                    sum += use ? q : 0ull;
                    mn = (use && q < mn) ? q : mn;
                }
            }
        }
        for (int d = LPB >> 1; d >= 1; d >>= 1) {  // xor shuffles stay inside the aligned group of LPB lanes
            sum += shfl_u64(sum, (tid & (kWave - 1)) ^ d);
            const unsigned long long o = shfl_u64(mn, (tid & (kWave - 1)) ^ d);
            mn = o < mn ? o : mn;
        }
        if (in && sub == 0) {
            const bool ok = ans >= 0 && len > 0;
            a[b] = ok ? ans : -1;
            w[b] = !ok ? 0.f
                       : (weight_mode == 0 ? (float)((double)mn / 1073741824.0)
                                           : (float)((double)sum / ((double)len * 1073741824.0)));
        }
    }
    __syncthreads();
    // selection: candidate i competes with key (score bits << 32) | (2^32 - 1 - i); scores are >= 0,
    // so their fp32 bit patterns order like the values, and equal scores go to the smaller index
    unsigned long long key = 0;
    for (int i = tid; i < B; i += kConfThreads) {
        if (a[i] < 0) continue;
        float score;
        if (select_mode == 0) {
            score = w[i];
        } else {
            bool first = true;
            for (int j = 0; j < i; ++j) first = first && !(a[j] == a[i]);
            if (!first) continue;
            score = 0.f;
            for (int j = 0; j < B; ++j)
                if (a[j] == a[i]) score = score + w[j];  // branch order, one rounding per add
        }
        const unsigned long long kk = ((unsigned long long)__float_as_uint(score) << 32) | (0xFFFFFFFFu - (unsigned)i);
        key = kk > key ? kk : key;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const unsigned long long o = shfl_down_u64(key, d);
        key = o > key ? o : key;
    }
    if ((tid & (kWave - 1)) == 0) sh_key[tid / kWave] = key;
    __syncthreads();
    if (tid == 0) {
        for (int i = 1; i < kConfThreads / kWave; ++i) key = sh_key[i] > key ? sh_key[i] : key;
        if (key == 0) {
            winner[n] = -1;
            winner_score[n] = 0.f;
        } else {
            winner[n] = a[0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFu)];
            winner_score[n] = __uint_as_float((unsigned)(key >> 32));
        }
    }
}

}  // namespace lotts

extern "C" int confidence_vote(int32_t N, int32_t B, int32_t T, const int32_t* answers, const float* conf,
                               const int32_t* conf_len, int32_t weight_mode, int32_t select_mode, int32_t* winner,
                               float* winner_score, void* stream) {
    if (!answers || !conf || !winner || !winner_score) return LOTTS_ERR_NULL;
    if (N < 1 || B < 1 || B > lotts::kConfMaxB || T < 1 || weight_mode < 0 || weight_mode > 1 || select_mode < 0 ||
        select_mode > 1)
        return LOTTS_ERR_SHAPE;
    LOTTS_LAUNCH(lotts::confidence_vote_kernel, dim3(N), dim3(lotts::kConfThreads), (hipStream_t)stream, B, T,
                       answers, conf, conf_len, weight_mode, select_mode, winner, winner_score);
    return lotts::check_launch();
}
