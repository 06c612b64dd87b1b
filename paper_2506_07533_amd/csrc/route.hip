// moqae_route_chunks: router MLP (Eq. (1), Sec. 3.2), token top-1 and chunk majority vote
// (Eq. (2)), routing freezing (Sec. 3.4).
//
// One wavefront per (sequence, KV head, chunk).  A lane owns one token: it requests its whole
// 256-byte key row at once (no LDS, no barrier in the loop) and runs
// the 2*M length-D dot products as sequential binary32 sums (the products of two fp16 values
// are exact in binary32, so a fused multiply-add rounds exactly like multiply-then-add), which
// is what makes the integer result reproducible bit for bit.  The router weights are
// wave-uniform: they are read through uniform 32-bit loads of the caller's fp16 arrays.
#include "moqae_dev.hpp"
#include "moqae_kernels.hpp"
#include "route_dev.hpp"

namespace moqae {

constexpr int kRouteThreads = 64;         // one wavefront per workgroup, one lane per token

template <int M>
__global__ __launch_bounds__(kRouteThreads) void route_kernel(RouteArgs a) {
    __shared__ float w3f[72];                        // W3 as binary32, then the optional bias

    const int c = a.chunk_begin + (int)blockIdx.x;
    const int u = (int)blockIdx.y;
    const int tid = (int)threadIdx.x;
    const int64_t eidx = (int64_t)u * a.expert_stride + c;

    if (c < a.freeze_chunks) {                       // routing freezing: never routed, FP16 expert
        if (tid == 0) a.expert[eidx] = (uint8_t)a.e16;
        if (a.votes && tid < M) a.votes[eidx * M + tid] = 0;
        return;
    }
    if (tid < M * M) w3f[tid] = half_bits_to_float(a.W3[tid]);
    if (a.bias && tid < M) w3f[64 + tid] = a.bias[tid];
    __syncthreads();

    const int b = u / a.Hkv, h = u % a.Hkv;
    const uint16_t *Kc = a.K + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h + (int64_t)c * a.N * a.stride_s;
    const uint32_t *W1w = reinterpret_cast<const uint32_t *>(a.W1);
    const uint32_t *W2w = reinterpret_cast<const uint32_t *>(a.W2);

    int cnt[M];                                      // votes, identical in every lane
    route_tokens<M>(Kc, a.N, a.stride_s, W1w, W2w, w3f, a.bias != nullptr, tid, cnt);
    if (tid == 0) {
        int best = 0, cbest = cnt[0];
#pragma unroll
        for (int k = 1; k < M; k++) if (cnt[k] > cbest) { best = k; cbest = cnt[k]; }
        a.expert[eidx] = (uint8_t)best;
    }
    if (a.votes) {
#pragma unroll
        for (int k = 0; k < M; k++) if (tid == k) a.votes[eidx * M + k] = cnt[k];
    }
}

template <int M>
static hipError_t launch_m(const RouteArgs &a, dim3 grid, hipStream_t s) {
    hipLaunchKernelGGL(route_kernel<M>, grid, dim3(kRouteThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_route(const RouteArgs &a, int M, int n_chunks, int BH, hipStream_t s) {
    if (n_chunks <= 0 || BH <= 0) return hipSuccess;
    dim3 grid((unsigned)n_chunks, (unsigned)BH);
    switch (M) {
        case 1: return launch_m<1>(a, grid, s);
        case 2: return launch_m<2>(a, grid, s);
        case 3: return launch_m<3>(a, grid, s);
        case 4: return launch_m<4>(a, grid, s);
        case 5: return launch_m<5>(a, grid, s);
        case 6: return launch_m<6>(a, grid, s);
        case 7: return launch_m<7>(a, grid, s);
        case 8: return launch_m<8>(a, grid, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace moqae
