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

namespace moqae {

// exp(x) with a fixed evaluation order: 2^n * P(r), t = x*log2(e), n = rint(t), r = t - n,
// P = degree-6 Taylor polynomial of 2^r in Horner form, every operation rounded separately.
__device__ __forceinline__ float exp_pinned(float x) {
    const float LOG2E = 0x1.715476p+0f;
    const float C1 = 0x1.62e430p-1f, C2 = 0x1.ebfbe0p-3f, C3 = 0x1.c6b08ep-5f;
    const float C4 = 0x1.3b2ab6p-7f, C5 = 0x1.5d87fep-10f, C6 = 0x1.430912p-13f;
    x = fminf(fmaxf(x, -80.0f), 80.0f);
    float t = __fmul_rn(x, LOG2E);
    float n = rintf(t);
    float r = __fsub_rn(t, n);
    float p = C6;
    p = __fadd_rn(__fmul_rn(p, r), C5);
    p = __fadd_rn(__fmul_rn(p, r), C4);
    p = __fadd_rn(__fmul_rn(p, r), C3);
    p = __fadd_rn(__fmul_rn(p, r), C2);
    p = __fadd_rn(__fmul_rn(p, r), C1);
    p = __fadd_rn(__fmul_rn(p, r), 1.0f);
    float s = __builtin_bit_cast(float, (uint32_t)((int)n + 127) << 23);
    return __fmul_rn(p, s);
}

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
#pragma unroll
    for (int k = 0; k < M; k++) cnt[k] = 0;

    float accA[M], accB[M];
    // The loop runs over half rows (64 dims = one 128-byte line per lane); the next half row is
    // requested before the current one is consumed, across the 64-token passes too.
    const int n_half = 2 * ((a.N + kRouteThreads - 1) / kRouteThreads);
    auto half_ptr = [&](int hr) {
        const int row = (hr >> 1) * kRouteThreads + tid;
        return reinterpret_cast<const uint4 *>(Kc + (int64_t)(row < a.N ? row : 0) * a.stride_s) + (hr & 1) * 8;
    };
    uint4 xn[8];
    {
        const uint4 *hp = half_ptr(0);
#pragma unroll
        for (int p = 0; p < 8; p++) xn[p] = hp[p];
    }
#pragma unroll 1
    for (int hr = 0; hr < n_half; hr++) {
        const int row0 = (hr >> 1) * kRouteThreads;
        const bool active = row0 + tid < a.N;        // N is a multiple of 32: the last pass may be half empty
        uint4 xr[8];
#pragma unroll
        for (int p = 0; p < 8; p++) xr[p] = xn[p];
        if (hr + 1 < n_half) {
            const uint4 *hp = half_ptr(hr + 1);
#pragma unroll
            for (int p = 0; p < 8; p++) xn[p] = hp[p];
        }
        if (!(hr & 1)) {
#pragma unroll
            for (int m = 0; m < M; m++) { accA[m] = 0.0f; accB[m] = 0.0f; }
        }
        // two key dims (two rows of the weight matrices) per step so that the fp16 pairs fall on 32-bit words
        const int dbase = (hr & 1) * 64;
#pragma unroll
        for (int p = 0; p < 8; p++) {
            const uint32_t xw[4] = {xr[p].x, xr[p].y, xr[p].z, xr[p].w};
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const int d = dbase + p * 8 + e;      // even; rows d, d+1 of W = 2*M halves = M words
                const float x0 = half_bits_to_float(xw[e >> 1] & 0xffffu);
                const float x1 = half_bits_to_float(xw[e >> 1] >> 16);
                uint32_t w1[M], w2[M];
#pragma unroll
                for (int m = 0; m < M; m++) { w1[m] = W1w[d / 2 * M + m]; w2[m] = W2w[d / 2 * M + m]; }
#pragma unroll
                for (int m = 0; m < M; m++) {
                    const int i0 = m, i1 = M + m;     // half index inside the two-row block
                    const float wa0 = half_bits_to_float((w1[i0 >> 1] >> (16 * (i0 & 1))) & 0xffffu);
                    const float wb0 = half_bits_to_float((w2[i0 >> 1] >> (16 * (i0 & 1))) & 0xffffu);
                    accA[m] = fmaf(x0, wa0, accA[m]);
                    accB[m] = fmaf(x0, wb0, accB[m]);
                    const float wa1 = half_bits_to_float((w1[i1 >> 1] >> (16 * (i1 & 1))) & 0xffffu);
                    const float wb1 = half_bits_to_float((w2[i1 >> 1] >> (16 * (i1 & 1))) & 0xffffu);
                    accA[m] = fmaf(x1, wa1, accA[m]);
                    accB[m] = fmaf(x1, wb1, accB[m]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);        // keeps the uniform weight loads of later steps from piling up
        }
        if (!(hr & 1)) continue;
        float hid[M];
#pragma unroll
        for (int m = 0; m < M; m++) {
            const float z = __fmul_rn(accA[m], accB[m]);
            const float e = exp_pinned(-z);
            hid[m] = __fdiv_rn(z, __fadd_rn(1.0f, e));              // SiLU(z) = z / (1 + exp(-z))
        }
        int top = 0; float ptop = 0.0f;
#pragma unroll
        for (int k = 0; k < M; k++) {
            float acc = 0.0f;
#pragma unroll
            for (int j = 0; j < M; j++) acc = __fadd_rn(acc, __fmul_rn(hid[j], w3f[j * M + k]));
            if (a.bias) acc = __fadd_rn(acc, w3f[64 + k]);
            if (k == 0) ptop = acc;
            else if (acc > ptop) { top = k; ptop = acc; }           // strict: the first maximum wins
        }
#pragma unroll
        for (int k = 0; k < M; k++) cnt[k] += __popcll(__ballot(active && top == k));
    }
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
