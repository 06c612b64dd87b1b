// Measurement aid (moqae_bench.h): a plain read-only streaming kernel.  What it reaches is the practical
// read ceiling of the chip, against which the decode kernel's share of the 8 TB/s HBM peak is read.
#include "../../include/moqae.h"
#include "../../include/moqae_bench.h"
#include <hip/hip_runtime.h>

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 8;                            // 16-byte loads in flight per lane
constexpr uint32_t kGroups = 256 * 8;                 // 8 workgroups of 4 wavefronts per compute unit

typedef uint32_t u4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kThreads) void stream_read_kernel(const u4 *__restrict__ src, uint64_t n16, uint32_t *__restrict__ sink) {
    __shared__ uint32_t red[kThreads / 64];
    u4 acc = {0u, 0u, 0u, 0u};
    const uint64_t span = (uint64_t)kThreads * kUnroll;                 // slots per workgroup and pass
    for (uint64_t base = (uint64_t)blockIdx.x * span; base < n16; base += (uint64_t)gridDim.x * span) {
        u4 v[kUnroll];
#pragma unroll
        for (int k = 0; k < kUnroll; k++) {
            const uint64_t i = base + (uint64_t)k * kThreads + threadIdx.x;   // a wavefront's load covers 1 KiB of consecutive bytes
            v[k] = i < n16 ? __builtin_nontemporal_load(src + i) : u4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int k = 0; k < kUnroll; k++) acc ^= v[k];
    }
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x ^= __shfl_xor(x, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = red[0] ^ red[1] ^ red[2] ^ red[3];
}

}  // namespace

extern "C" {

uint32_t moqae_bench_stream_sink_words(void) { return kGroups; }

int moqae_bench_stream_read(const void *buf, uint64_t bytes, uint32_t *sink, void *stream) {
    if (!buf || !sink || bytes == 0 || bytes % 16 || (reinterpret_cast<uintptr_t>(buf) & 15)) return MOQAE_E_INVAL;
    hipLaunchKernelGGL(stream_read_kernel, dim3(kGroups), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u4 *>(buf), bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

}  // extern "C"
