// moqae_router_loss_grad: the router fine-tuning loss of Sec. 3.3 (Eq. (3)-(5)) and its gradient with respect to
// the router weights, over cached key rows, in one pass.
//
//   L = (1/T) sum_i p^i_j * (lambda * L_nll * pen_model_j + (1 - lambda) * pen_mem_j),  j = the token's top-1 expert,
//   p^i = softmax of the token's logits.  The top-1 index comes from the same binary32 arithmetic as routing
//   (route_kernel), so it is the routing decision bit for bit; everything after it is plain binary32.
//
// One wavefront per tile of 64 tokens, one lane per token for the forward pass and the token's own backward
// pass down to d(loss)/d(xW1), d(loss)/d(xW2) (2M values per token, handed over through LDS); then the lane
// owning dims (2l, 2l+1) adds x[t][d] * d.. over the tile's tokens into dW1, dW2 accumulators that stay in
// registers for all tiles of the wavefront (the rows come back from L2 as coalesced 256-byte reads).  dW3, the
// bias gradient and the loss are per-lane sums folded at the end.  Bound by the vector ALU: about 2 * 2M * D
// multiply-adds per token forward and as many backward.
#include "moqae_dev.hpp"
#include "moqae_kernels.hpp"
#include "route_dev.hpp"

namespace moqae {

constexpr int kTrainWaves = 4;

template <int M>
__global__ __launch_bounds__(kTrainWaves * 64) void router_train_kernel(TrainArgs a) {
    __shared__ float w3f[72];
    __shared__ float dab[kTrainWaves][64][2 * M];     // per token: d/d(xW1)[M], d/d(xW2)[M]
    __shared__ float red[kTrainWaves][4 * M * 64];    // dW1, dW2 of the wavefronts at the end
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < M * M) w3f[tid] = half_bits_to_float(a.W3[tid]);
    if (tid < M) w3f[64 + tid] = a.bias ? a.bias[tid] : 0.0f;
    __syncthreads();
    const uint32_t *W1w = reinterpret_cast<const uint32_t *>(a.W1);
    const uint32_t *W2w = reinterpret_cast<const uint32_t *>(a.W2);

    float g1[2][M], g2[2][M];                         // dW1[2l + e][m], dW2[2l + e][m]
    float g3[M][M], gb[M], lsum[2] = {0.0f, 0.0f};
#pragma unroll
    for (int m = 0; m < M; m++) {
        g1[0][m] = g1[1][m] = g2[0][m] = g2[1][m] = 0.0f; gb[m] = 0.0f;
#pragma unroll
        for (int k = 0; k < M; k++) g3[m][k] = 0.0f;
    }
    const int tiles_per_row = (a.n_tok + 63) / 64;
    const long long n_tiles = (long long)a.BH * tiles_per_row;
    const long long gw = (long long)blockIdx.x * kTrainWaves + wave, tw = (long long)gridDim.x * kTrainWaves;
    for (long long tile = gw; tile < n_tiles; tile += tw) {
        const int u = (int)(tile / tiles_per_row), t0 = (int)(tile % tiles_per_row) * 64;
        const int b = u / a.Hkv, h = u % a.Hkv;
        const int n_here = min(64, a.n_tok - t0);
        const bool active = lane < n_here;
        const uint16_t *Kt = a.K + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h + (int64_t)(a.token_begin + t0) * a.stride_s;
        // ---- forward, the routing arithmetic: sequential binary32 sums over d (products of two fp16 values are exact)
        float accA[M], accB[M];
#pragma unroll
        for (int m = 0; m < M; m++) { accA[m] = 0.0f; accB[m] = 0.0f; }
        const uint4 *rowp = reinterpret_cast<const uint4 *>(Kt + (int64_t)(active ? lane : 0) * a.stride_s);
#pragma unroll 1
        for (int hr = 0; hr < 2; hr++) {
            uint4 xr[8];
#pragma unroll
            for (int p = 0; p < 8; p++) xr[p] = rowp[hr * 8 + p];
#pragma unroll
            for (int p = 0; p < 8; p++) {
                const uint32_t xw[4] = {xr[p].x, xr[p].y, xr[p].z, xr[p].w};
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const int d = hr * 64 + p * 8 + e;
                    const float x0 = half_bits_to_float(xw[e >> 1] & 0xffffu), x1 = half_bits_to_float(xw[e >> 1] >> 16);
                    uint32_t w1[M], w2[M];
#pragma unroll
                    for (int m = 0; m < M; m++) { w1[m] = W1w[d / 2 * M + m]; w2[m] = W2w[d / 2 * M + m]; }
#pragma unroll
                    for (int m = 0; m < M; m++) {
                        const int i0 = m, i1 = M + m;
                        accA[m] = fmaf(x0, half_bits_to_float((w1[i0 >> 1] >> (16 * (i0 & 1))) & 0xffffu), accA[m]);
                        accB[m] = fmaf(x0, half_bits_to_float((w2[i0 >> 1] >> (16 * (i0 & 1))) & 0xffffu), accB[m]);
                        accA[m] = fmaf(x1, half_bits_to_float((w1[i1 >> 1] >> (16 * (i1 & 1))) & 0xffffu), accA[m]);
                        accB[m] = fmaf(x1, half_bits_to_float((w2[i1 >> 1] >> (16 * (i1 & 1))) & 0xffffu), accB[m]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        float z[M], sg[M], hid[M], lg[M];
#pragma unroll
        for (int m = 0; m < M; m++) {
            z[m] = __fmul_rn(accA[m], accB[m]);
            const float den = __fadd_rn(1.0f, exp_pinned(-z[m]));
            hid[m] = __fdiv_rn(z[m], den);
            sg[m] = 1.0f / den;
        }
        int top = 0;
#pragma unroll
        for (int k = 0; k < M; k++) {
            float acc = 0.0f;
#pragma unroll
            for (int j = 0; j < M; j++) acc = __fadd_rn(acc, __fmul_rn(hid[j], w3f[j * M + k]));
            if (a.bias) acc = __fadd_rn(acc, w3f[64 + k]);
            lg[k] = acc;
            if (k > 0 && acc > lg[top]) top = k;       // strict: the first maximum wins
        }
        // ---- loss of the token and its gradient down to xW1, xW2
        float mx = lg[0];
#pragma unroll
        for (int k = 1; k < M; k++) mx = fmaxf(mx, lg[k]);
        float p[M], den = 0.0f;
#pragma unroll
        for (int k = 0; k < M; k++) { p[k] = __expf(lg[k] - mx); den += p[k]; }
        const float rden = 1.0f / den;
        float ptop = 0.0f, pm = 0.0f, pe = 0.0f;
#pragma unroll
        for (int k = 0; k < M; k++) { p[k] *= rden; if (k == top) { ptop = p[k]; pm = a.pen_model[k]; pe = a.pen_mem[k]; } }
        const float nll = a.nll[b];
        const float act = active ? 1.0f : 0.0f;
        lsum[0] += act * ptop * nll * pm; lsum[1] += act * ptop * pe;
        const float w = act * (a.lambda * nll * pm + (1.0f - a.lambda) * pe) * ptop * a.inv_T;
        float dl[M];
#pragma unroll
        for (int k = 0; k < M; k++) { dl[k] = w * ((k == top ? 1.0f : 0.0f) - p[k]); gb[k] += dl[k]; }
        float dxa[M], dxb[M];
#pragma unroll
        for (int m = 0; m < M; m++) {
            float dh = 0.0f;
#pragma unroll
            for (int k = 0; k < M; k++) { dh = fmaf(dl[k], w3f[m * M + k], dh); g3[m][k] = fmaf(hid[m], dl[k], g3[m][k]); }
            const float dz = dh * (sg[m] * (1.0f + z[m] * (1.0f - sg[m])));
            dxa[m] = dz * accB[m]; dxb[m] = dz * accA[m];
        }
#pragma unroll
        for (int m = 0; m < M; m++) { dab[wave][lane][m] = dxa[m]; dab[wave][lane][M + m] = dxb[m]; }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // ---- dW1, dW2: this lane's two dims over the tile's tokens (rows re-read as coalesced 256-byte pieces)
        const uint32_t *colp = reinterpret_cast<const uint32_t *>(Kt) + lane;
#pragma unroll 1
        for (int tb = 0; tb < 64; tb += 8) {
            uint32_t xw[8];
#pragma unroll
            for (int i = 0; i < 8; i++) xw[i] = colp[(int64_t)min(tb + i, n_here - 1) * (a.stride_s / 2)];
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const float x0 = half_bits_to_float(xw[i] & 0xffffu), x1 = half_bits_to_float(xw[i] >> 16);
#pragma unroll
                for (int m = 0; m < M; m++) {
                    const float da = dab[wave][tb + i][m], db = dab[wave][tb + i][M + m];   // zero for tokens past the tile's end
                    g1[0][m] = fmaf(x0, da, g1[0][m]); g1[1][m] = fmaf(x1, da, g1[1][m]);
                    g2[0][m] = fmaf(x0, db, g2[0][m]); g2[1][m] = fmaf(x1, db, g2[1][m]);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    // ---- fold: per-lane sums over the wavefront, the wavefronts over the workgroup, the workgroups by atomic adds
    auto wsum = [](float v) {
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
        return v;
    };
#pragma unroll
    for (int m = 0; m < M; m++) {
#pragma unroll
        for (int k = 0; k < M; k++) { const float v = wsum(g3[m][k]); if (lane == 0) atomicAdd(&a.dW3[m * M + k], v); }
        const float v = wsum(gb[m]);
        if (lane == 0 && a.dbias) atomicAdd(&a.dbias[m], v);
    }
    {
        const float lm = wsum(lsum[0]) * a.inv_T, le = wsum(lsum[1]) * a.inv_T;
        if (lane == 0) {
            atomicAdd(&a.loss3[1], lm); atomicAdd(&a.loss3[2], le);
            atomicAdd(&a.loss3[0], a.lambda * lm + (1.0f - a.lambda) * le);
        }
    }
#pragma unroll
    for (int e = 0; e < 2; e++) {
#pragma unroll
        for (int m = 0; m < M; m++) {
            red[wave][((2 * lane + e) * M + m)] = g1[e][m];
            red[wave][2 * M * 64 + ((2 * lane + e) * M + m)] = g2[e][m];
        }
    }
    __syncthreads();
    for (int i = tid; i < 4 * M * 64; i += kTrainWaves * 64) {
        float v = 0.0f;
#pragma unroll
        for (int wv = 0; wv < kTrainWaves; wv++) v += red[wv][i];
        if (i < 2 * M * 64) atomicAdd(&a.dW1[i], v); else atomicAdd(&a.dW2[i - 2 * M * 64], v);
    }
}

__global__ void train_zero_kernel(TrainArgs a) {
    const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (i < kD * a.M) { a.dW1[i] = 0.0f; a.dW2[i] = 0.0f; }
    if (i < a.M * a.M) a.dW3[i] = 0.0f;
    if (i < a.M && a.dbias) a.dbias[i] = 0.0f;
    if (i < 3) a.loss3[i] = 0.0f;
}

template <int M>
static hipError_t launch_t(const TrainArgs &a, unsigned n_wg, hipStream_t s) {
    hipLaunchKernelGGL(router_train_kernel<M>, dim3(n_wg), dim3(kTrainWaves * 64), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_router_train(const TrainArgs &a, int n_cu, hipStream_t s) {
    hipLaunchKernelGGL(train_zero_kernel, dim3((kD * 8 + 255) / 256), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long n_tiles = (long long)a.BH * ((a.n_tok + 63) / 64);
    long long n_wg = (n_tiles + kTrainWaves - 1) / kTrainWaves;
    if (n_wg > 4LL * n_cu) n_wg = 4LL * n_cu;          // every wavefront keeps its dW accumulators over many tiles
    switch (a.M) {
        case 1: return launch_t<1>(a, (unsigned)n_wg, s);
        case 2: return launch_t<2>(a, (unsigned)n_wg, s);
        case 3: return launch_t<3>(a, (unsigned)n_wg, s);
        case 4: return launch_t<4>(a, (unsigned)n_wg, s);
        case 5: return launch_t<5>(a, (unsigned)n_wg, s);
        case 6: return launch_t<6>(a, (unsigned)n_wg, s);
        case 7: return launch_t<7>(a, (unsigned)n_wg, s);
        case 8: return launch_t<8>(a, (unsigned)n_wg, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace moqae
