// Device code of the router shared by route_kernel and the fused route + pack kernel (Eq. (1)-(2), Sec. 3.2).
#pragma once
#include "moqae_dev.hpp"

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

// 64 dims of a key row (eight 16-byte pieces xr[0..7], dims dbase..dbase+63) into the two running sums per expert,
// in ascending order of the dims.  W1w, W2w: the fp16 weight matrices as 32-bit words (wave-uniform loads).
template <int M>
__device__ __forceinline__ void route_half_row(const uint4 *xr, int dbase, const uint32_t *W1w, const uint32_t *W2w,
                                               float (&accA)[M], float (&accB)[M]) {
    // two key dims (two rows of the weight matrices) per step so that the fp16 pairs fall on 32-bit words
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
}

// The token's expert from the two sums per expert: SiLU of their product, times W3 (plus the bias), first maximum.
// w3f: W3 as binary32 (M*M values) and the optional bias at [64..64+M), in LDS.
template <int M>
__device__ __forceinline__ int route_top(const float (&accA)[M], const float (&accB)[M], const float *w3f, bool has_bias) {
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
        if (has_bias) acc = __fadd_rn(acc, w3f[64 + k]);
        if (k == 0) ptop = acc;
        else if (acc > ptop) { top = k; ptop = acc; }           // strict: the first maximum wins
    }
    return top;
}

// One token's expert from its whole key row in registers (sixteen 16-byte pieces): the same operations in the same
// order as route_tokens.
template <int M>
__device__ __forceinline__ int route_row(const uint4 (&x)[16], const uint32_t *W1w, const uint32_t *W2w, const float *w3f,
                                         bool has_bias) {
    float accA[M], accB[M];
#pragma unroll
    for (int m = 0; m < M; m++) { accA[m] = 0.0f; accB[m] = 0.0f; }
    route_half_row<M>(&x[0], 0, W1w, W2w, accA, accB);
    route_half_row<M>(&x[8], 64, W1w, W2w, accA, accB);
    return route_top<M>(accA, accB, w3f, has_bias);
}

// One wavefront routes the n_tok tokens whose key rows start at Kc (row stride stride_s elements), one lane per
// token and pass of 64 tokens; W1w, W2w: the fp16 weight matrices as 32-bit words (wave-uniform loads), w3f: W3 as
// binary32 (M*M values) and the optional bias at [64..64+M), in LDS.  Returns the votes per expert, the same in
// every lane.  STAGE: every lane also leaves its rows in `stage` (LDS, kStageRow 16-byte pieces per row, row = token
// counted from Kc), so that a quantiser that follows reads the keys from there and not from memory again.
constexpr int kStageRow = 17;                     // 16 pieces of data + 1 of padding: the lanes' writes fall on different banks
template <int M, bool STAGE = false>
__device__ __forceinline__ void route_tokens(const uint16_t *Kc, int n_tok, int64_t stride_s, const uint32_t *W1w,
                                             const uint32_t *W2w, const float *w3f, bool has_bias, int lane, int (&cnt)[M],
                                             uint4 *stage = nullptr) {
#pragma unroll
    for (int k = 0; k < M; k++) cnt[k] = 0;

    float accA[M], accB[M];
    // The loop runs over half rows (64 dims = one 128-byte line per lane); the next half row is
    // requested before the current one is consumed, across the 64-token passes too.
    const int n_half = 2 * ((n_tok + 64 - 1) / 64);
    auto half_ptr = [&](int hr) {
        const int row = (hr >> 1) * 64 + lane;
        return reinterpret_cast<const uint4 *>(Kc + (int64_t)(row < n_tok ? row : 0) * stride_s) + (hr & 1) * 8;
    };
    uint4 xn[8];
    {
        const uint4 *hp = half_ptr(0);
#pragma unroll
        for (int p = 0; p < 8; p++) xn[p] = hp[p];
    }
#pragma unroll 1
    for (int hr = 0; hr < n_half; hr++) {
        const int row0 = (hr >> 1) * 64;
        const bool active = row0 + lane < n_tok;        // the last pass may be partly empty
        uint4 xr[8];
#pragma unroll
        for (int p = 0; p < 8; p++) xr[p] = xn[p];
        if constexpr (STAGE) {
            if (active) {
#pragma unroll
                for (int p = 0; p < 8; p++) stage[(row0 + lane) * kStageRow + (hr & 1) * 8 + p] = xr[p];
            }
        }
        if (hr + 1 < n_half) {
            const uint4 *hp = half_ptr(hr + 1);
#pragma unroll
            for (int p = 0; p < 8; p++) xn[p] = hp[p];
        }
        if (!(hr & 1)) {
#pragma unroll
            for (int m = 0; m < M; m++) { accA[m] = 0.0f; accB[m] = 0.0f; }
        }
        route_half_row<M>(xr, (hr & 1) * 64, W1w, W2w, accA, accB);
        if (!(hr & 1)) continue;
        const int top = route_top<M>(accA, accB, w3f, has_bias);
#pragma unroll
        for (int k = 0; k < M; k++) cnt[k] += __popcll(__ballot(active && top == k));
    }
}

}  // namespace moqae
