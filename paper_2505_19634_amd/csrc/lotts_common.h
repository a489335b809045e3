// Shared by the HIP translation units of liblotts.so: status codes, launch checking and
// wavefront helpers.  gfx950 only (64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include "lotts.h"

namespace lotts {

constexpr int kWave = 64;
// MI355X: 256 compute units in 8 XCDs.  Launch plans are sized for this part and do not depend
// on the device the process happens to see, so workspace queries agree everywhere.
constexpr int kNumCU = 256;
constexpr int kNumXCD = 8;

// Kernel timer (lotts_timer_start / lotts_timer_stop, kernel_timer.hip).  While it runs on the calling
// host thread, timer_take hands out one pair of events per launch and the launch carries them, so
// the pair reads that kernel's own start and end on the device.
bool timer_take(hipEvent_t* start, hipEvent_t* stop);

// Tag of a call whose workgroups exchange tagged words through the workspace (spec_accept,
// spec_accept_logits): never 0, and different for every such call of the process whichever entry point
// makes it, so one buffer can serve both without either taking the other's leftovers for its own.
unsigned next_word_tag();

// Every launch of the library goes through here: no dynamic LDS, the caller's stream.
#define LOTTS_LAUNCH(kernel, grid, block, stream, ...)                                                        \
    do {                                                                                                      \
        hipEvent_t lotts_e0_, lotts_e1_;                                                                      \
        if (lotts::timer_take(&lotts_e0_, &lotts_e1_))                                                        \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, lotts_e0_, lotts_e1_, 0, __VA_ARGS__);     \
        else                                                                                                  \
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);                                  \
    } while (0)

inline int check_launch() {
    return hipGetLastError() == hipSuccess ? LOTTS_OK : LOTTS_ERR_LAUNCH;
}

__device__ __forceinline__ float shfl_xor_f(float v, int mask) { return __shfl_xor(v, mask, kWave); }

__device__ __forceinline__ unsigned long long shfl_down_u64(unsigned long long v, int delta) {
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    lo = __shfl_down(lo, delta, kWave);
    hi = __shfl_down(hi, delta, kWave);
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned long long shfl_up_u64(unsigned long long v, int delta) {
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    lo = __shfl_up(lo, delta, kWave);
    hi = __shfl_up(hi, delta, kWave);
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned long long shfl_u64(unsigned long long v, int src) {
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    lo = __shfl(lo, src, kWave);
    hi = __shfl(hi, src, kWave);
    return ((unsigned long long)hi << 32) | lo;
}
// sum over the wavefront; the total is valid in lane 0
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += shfl_down_u64(v, d);
    return v;
}
// inclusive prefix sum over the wavefront
__device__ __forceinline__ unsigned long long wave_incl_scan_u64(unsigned long long v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        unsigned long long o = shfl_up_u64(v, d);
        if (lane >= d) v += o;
    }
    return v;
}

}  // namespace lotts
