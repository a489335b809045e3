// majority_vote: the answer most branches give (paper Section 1 / Section 4.1: branches are
// aggregated by majority voting).  One workgroup per question; B is tens to a few thousand
// ids, so this is a latency-bound O(B^2 / 256) count in LDS -- or, for up to 64 branches, in the
// lanes of a single wavefront.
#include "lotts_common.h"

namespace lotts {

constexpr int kVoteThreads = 256;
constexpr int kVoteMaxB = 4096;

__global__ __launch_bounds__(kVoteThreads) void majority_vote_kernel(int B, const int32_t* __restrict__ answers,
                                                                     int32_t* __restrict__ winner,
                                                                     int32_t* __restrict__ winner_count) {
    __shared__ int32_t a[kVoteMaxB];
    __shared__ unsigned long long best[kVoteThreads / kWave];
    const int n = blockIdx.x, tid = threadIdx.x;
    const int32_t* row = answers + (size_t)n * B;
    for (int i = tid; i < B; i += kVoteThreads) a[i] = row[i];
    __syncthreads();
    // Only the first occurrence of an id competes.  Key = (votes << 32) | (2^32 - 1 - index):
    // the maximum is the largest vote count, and among equal counts the smallest index.
    unsigned long long key = 0;
    for (int i = tid; i < B; i += kVoteThreads) {
        const int32_t ai = a[i];
        if (ai < 0) continue;
        int votes = 0;
        bool first = true;
        for (int j = 0; j < B; ++j) {
            const bool same = (a[j] == ai);
            votes += same;
            first = first && !(same && j < i);
        }
        if (first) {
            const unsigned long long kk = ((unsigned long long)votes << 32) | (0xFFFFFFFFu - (unsigned)i);
            key = kk > key ? kk : key;
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const unsigned long long o = shfl_down_u64(key, d);
        key = o > key ? o : key;
    }
    if ((tid & (kWave - 1)) == 0) best[tid / kWave] = key;
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kVoteThreads / kWave; ++w) key = best[w] > key ? best[w] : key;
        if (key == 0) {
            winner[n] = -1;
            winner_count[n] = 0;
        } else {
            winner[n] = a[0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFu)];
            winner_count[n] = (int32_t)(key >> 32);
        }
    }
}

// Up to 64 answers (the paper's branch counts): one wavefront, one answer per lane, no LDS, no barrier and
// no cross-lane data movement beyond reading one lane at a time: for every lane j in turn the wavefront
// compares its answers with answer j in one instruction, and the resulting lane mask -- a scalar -- gives the
// id's vote count (its population count) and tells whether j is the id's first occurrence (its lowest set bit).
// The whole kernel is one load, B compares with scalar bookkeeping, and one store.
__global__ __launch_bounds__(kWave) void majority_vote_wave_kernel(int B, const int32_t* __restrict__ answers,
                                                                   int32_t* __restrict__ winner,
                                                                   int32_t* __restrict__ winner_count) {
    const int n = blockIdx.x, lane = threadIdx.x;
    __builtin_assume(B >= 1);  // checked on the host; lets all arguments be fetched in one go
    // every lane loads (lanes past B re-read the last answer): with the load under a branch on B the pointer would
    // only be fetched after B has arrived and been compared -- one more dependent trip to the argument block
    const int32_t av = answers[(size_t)n * B + (lane < B ? lane : B - 1)];
    const int32_t ai = lane < B ? av : -1;
    int best = 0;
    int32_t best_a = -1;
    for (int j = 0; j < B; ++j) {  // everything in this loop is uniform over the wavefront
        const int32_t aj = __builtin_amdgcn_readlane(ai, j);
        if (aj < 0) continue;  // "no answer" does not compete
        const unsigned long long same = __ballot(ai == aj);
        if (__ffsll((long long)same) - 1 != j) continue;  // a later occurrence: the id has competed already
        const int votes = __popcll(same);
        if (votes > best) {  // strictly more: of equal counts the earlier first occurrence stays
            best = votes;
            best_a = aj;
        }
    }
    if (lane == 0) {
        winner[n] = best_a;
        winner_count[n] = best;
    }
}

}  // namespace lotts

extern "C" int majority_vote(int32_t N, int32_t B, const int32_t* answers, int32_t* winner, int32_t* winner_count,
                             void* stream) {
    if (!answers || !winner || !winner_count) return LOTTS_ERR_NULL;
    if (N < 1 || B < 1 || B > lotts::kVoteMaxB) return LOTTS_ERR_SHAPE;
    if (B <= lotts::kWave)
        LOTTS_LAUNCH(lotts::majority_vote_wave_kernel, dim3(N), dim3(lotts::kWave), (hipStream_t)stream, B, answers,
                     winner, winner_count);
    else
        LOTTS_LAUNCH(lotts::majority_vote_kernel, dim3(N), dim3(lotts::kVoteThreads), (hipStream_t)stream, B, answers,
                     winner, winner_count);
    return lotts::check_launch();
}

extern "C" const char* lotts_strerror(int status) {
    switch (status) {
        case LOTTS_OK: return "ok";
        case LOTTS_ERR_NULL: return "a required pointer is NULL";
        case LOTTS_ERR_SHAPE: return "unsupported sizes, strides or alignment";
        case LOTTS_ERR_DTYPE: return "unsupported element type";
        case LOTTS_ERR_WORKSPACE: return "workspace too small";
        case LOTTS_ERR_LAUNCH: return "HIP launch failed";
        default: return "unknown lotts status";
    }
}
