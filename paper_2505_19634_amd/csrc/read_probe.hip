// read_probe: a read-only streaming kernel over two device buffers, timed like the library's own
// launches (an event pair attached to the dispatch).  Its only use is to put a ceiling next to the
// attention kernel's bandwidth figure: what a kernel that does nothing but read the same bytes
// reaches on the same box, with the same launch shape (256 workgroups of 4 wavefronts, one per
// compute unit; every wavefront keeps 16 non-temporal 16-byte loads per lane in flight: 8 KB from
// each buffer, the size of one K and one V tile).  Measurement aid: built as libread_probe.so, not
// part of liblotts.so.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256, kWave = 64, kGroups = 256;
constexpr int kPiece = 8192;  // bytes a wavefront takes from each buffer per step

__global__ __launch_bounds__(kThreads) void read_probe_kernel(const char* __restrict__ a, const char* __restrict__ b,
                                                              size_t pieces, unsigned* __restrict__ sink) {
    const int lane = threadIdx.x & (kWave - 1);
    const size_t wave = (size_t)blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
    const size_t waves = (size_t)gridDim.x * (kThreads / kWave);
    unsigned acc = 0;
    // pieces are dealt round-robin to all wavefronts, so neighbouring wavefronts read neighbouring memory
    for (size_t p = wave; p < pieces; p += waves) {
        u32x4 va[8], vb[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const size_t off = p * kPiece + (size_t)i * 1024 + (size_t)lane * 16;
            va[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(a + off));
            vb[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(b + off));
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) acc += (va[i].x ^ va[i].y ^ va[i].z ^ va[i].w) + (vb[i].x ^ vb[i].y ^ vb[i].z ^ vb[i].w);
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;  // keeps the loads alive; practically never taken
}

hipEvent_t g_start = nullptr, g_stop = nullptr;

}  // namespace

// Reads bytes_each bytes (rounded down to a multiple of 8192) from each of the device buffers a and b
// once, on `stream`, and returns the kernel's device time in milliseconds in *ms (the call waits for
// the kernel).  sink: 4 bytes of device memory.  Returns 0, or -1 on a bad argument / HIP error.
extern "C" int read_probe(const void* a, const void* b, size_t bytes_each, void* sink, void* stream, float* ms) {
    if (!a || !b || !sink || !ms || bytes_each < kPiece) return -1;
    if (!g_start && (hipEventCreate(&g_start) != hipSuccess || hipEventCreate(&g_stop) != hipSuccess)) return -1;
    hipExtLaunchKernelGGL(read_probe_kernel, dim3(kGroups), dim3(kThreads), 0, (hipStream_t)stream, g_start, g_stop, 0,
                          static_cast<const char*>(a), static_cast<const char*>(b), bytes_each / kPiece,
                          static_cast<unsigned*>(sink));
    if (hipGetLastError() != hipSuccess) return -1;
    if (hipEventSynchronize(g_stop) != hipSuccess) return -1;
    return hipEventElapsedTime(ms, g_start, g_stop) == hipSuccess ? 0 : -1;
}
