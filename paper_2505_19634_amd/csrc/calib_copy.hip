// calib_copy: a plain device-to-device copy kernel of known size.  Its only use is to calibrate
// the HBM traffic counters (FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc): the factor between
// what a counter reads for this kernel and the bytes it is known to move is applied to the
// counter readings of the attention kernel.  Not part of liblotts.so.
//
//   calib_copy [MiB per copy = 256] [launches = 12]
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            std::fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));       \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}

int main(int argc, char** argv) {
    const size_t mib = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 256;
    const int launches = argc > 2 ? std::atoi(argv[2]) : 12;
    const size_t bytes = mib << 20;
    const int nsets = 4;  // rotate so that the memory-side cache cannot serve the reads
    char* buf = nullptr;
    CHECK(hipMalloc(&buf, bytes * nsets * 2));
    CHECK(hipMemset(buf, 1, bytes * nsets * 2));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    float total_ms = 0.f;
    for (int it = 0; it < launches; ++it) {
        const uint4* src = reinterpret_cast<const uint4*>(buf + (size_t)(it % nsets) * 2 * bytes);
        uint4* dst = reinterpret_cast<uint4*>(buf + ((size_t)(it % nsets) * 2 + 1) * bytes);
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL(calib_copy_kernel, dim3(4096), dim3(256), 0, 0, src, dst, bytes / 16);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms = 0.f;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        total_ms += ms;
    }
    std::printf("calib_copy: %d launches, %zu bytes read + %zu bytes written per launch, avg %.1f us (%.0f GB/s read+write)\n",
                launches, bytes, bytes, total_ms / launches * 1e3, 2.0 * bytes / (total_ms / launches * 1e-3) / 1e9);
    CHECK(hipFree(buf));
    return 0;
}
