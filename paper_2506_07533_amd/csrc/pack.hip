// moqae_quantize_pack: offset plan + group-wise quantisation and bit-packing of every chunk
// at its routed bit-width (Sec. 3.1-3.2 of the paper say only that a chunk is quantised with
// the configuration its router chose; the quantiser and the layout are defined in moqae.h).
//
//   plan_kernel  one workgroup: block sizes -> exclusive scan in (b, h, c) order -> offsets,
//                capacity check, new arena end.
//   pack_kernel  one workgroup per (chunk, K or V).  16 lanes own one token row (8 dims each),
//                group min/max by DPP, codes in registers.  K words are assembled in registers
//                (row-major layout); V codes go through LDS as bytes and are gathered
//                token-wise into the dimension-major tile layout.  HBM-bound: reads 2*N*D*2 bytes,
//                writes the block.
#include "moqae_dev.hpp"
#include "moqae_kernels.hpp"

namespace moqae {

constexpr int kPlanThreads = 1024;

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(PackArgs a) {
    __shared__ unsigned long long scan[kPlanThreads];
    __shared__ int bad;
    const int tid = (int)threadIdx.x;
    if (*a.status != 0) return;                       // sticky error: the call is a no-op
    if (tid == 0) bad = 0;
    __syncthreads();

    const int64_t total = (int64_t)a.BH * a.n_chunks;
    const int64_t per = (total + kPlanThreads - 1) / kPlanThreads;
    const int64_t i0 = min(total, per * tid), i1 = min(total, i0 + per);
    const int64_t u0 = i0 / a.n_chunks; const int cc0 = (int)(i0 % a.n_chunks);
    unsigned long long size_of[8];                    // rounded block size per expert
#pragma unroll
    for (int e = 0; e < 8; e++) size_of[e] = (block_bytes(a.N, a.G, a.bits_of[e]) + 255u) & ~255ull;
    auto size_at = [&](int e) {
        unsigned long long v = 0;
#pragma unroll
        for (int k = 0; k < 8; k++) v = (e == k) ? size_of[k] : v;
        return v;
    };
    unsigned long long local = 0;
    {
        int64_t u = u0; int cc = cc0;
        for (int64_t i = i0; i < i1; i += 8) {            // eight independent loads in flight
            int e[8];
#pragma unroll
            for (int k = 0; k < 8; k++) {
                e[k] = (i + k < i1) ? a.expert[u * a.expert_stride + a.chunk_begin + cc] : 0;
                if (++cc == a.n_chunks) { cc = 0; u++; }
            }
#pragma unroll
            for (int k = 0; k < 8; k++) if (i + k < i1) { if (e[k] >= a.M) bad = 1; else local += size_at(e[k]); }
        }
    }
    scan[tid] = local;
    __syncthreads();
    for (int off = 1; off < kPlanThreads; off <<= 1) {          // Hillis-Steele inclusive scan
        unsigned long long v = tid >= off ? scan[tid - off] : 0;
        __syncthreads();
        scan[tid] += v;
        __syncthreads();
    }
    const unsigned long long start = (*a.arena_used + 255u) & ~255ull;
    const unsigned long long sum = scan[kPlanThreads - 1];
    if (bad) { if (tid == 0) *a.status = -1; return; }
    if (start + sum > a.capacity) { if (tid == 0) *a.status = -3; return; }
    unsigned long long pos = start + scan[tid] - local;
    {
        int64_t u = u0; int cc = cc0;
        for (int64_t i = i0; i < i1; i += 8) {
            int e[8]; int64_t at[8];
#pragma unroll
            for (int k = 0; k < 8; k++) {
                at[k] = u * a.off_stride + a.chunk_begin + cc;
                e[k] = (i + k < i1) ? a.expert[u * a.expert_stride + a.chunk_begin + cc] : 0;
                if (++cc == a.n_chunks) { cc = 0; u++; }
            }
#pragma unroll
            for (int k = 0; k < 8; k++) if (i + k < i1) { a.chunk_off[at[k]] = pos; pos += size_at(e[k]); }
        }
    }
    __syncthreads();                                  // every thread has read *arena_used
    if (tid == 0) *a.arena_used = start + sum;
}

constexpr int kPackThreads = 256;

// Position of the code with in-word index e (b bits): even e in the low half-word, odd e high.
__device__ __forceinline__ int code_shift(int e, int b) { return 16 * (e & 1) + b * (e >> 1); }

template <int G>
__global__ __launch_bounds__(kPackThreads) void pack_kernel(PackArgs a) {
    extern __shared__ uint8_t vcodes[];               // [N][128] code bytes (V only)
    if (*a.status != 0) return;

    const int c = a.chunk_begin + (int)blockIdx.x;
    const int u = (int)blockIdx.y;
    const int isV = (int)blockIdx.z;
    const int tid = (int)threadIdx.x;
    const int N = a.N;
    const int bits = a.bits_of[a.expert[(int64_t)u * a.expert_stride + c]];
    uint8_t *blk = a.arena + a.chunk_off[(int64_t)u * a.off_stride + c];
    const int b = u / a.Hkv, h = u % a.Hkv;
    const uint16_t *src = (isV ? a.V : a.K) + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h
                        + (int64_t)c * N * a.stride_s;
    const int lane16 = tid & 15;                      // which 8 dims of the row
    const int rsub = tid >> 4;                        // row inside a pass of 16 rows

    if (bits == 16) {                                 // FP16 expert: rows copied verbatim
        uint4 *dst = reinterpret_cast<uint4 *>(blk + (isV ? (size_t)N * kD * 2 : 0));
        for (int row = rsub; row < N; row += kPackThreads / 16)
            dst[row * 16 + lane16] = *reinterpret_cast<const uint4 *>(src + (int64_t)row * a.stride_s + lane16 * 8);
        return;
    }

    constexpr int NG = kD / G;                        // groups per row
    constexpr int LPG = G / 8;                        // lanes per group
    const size_t code_bytes = (size_t)N * kD * bits / 8, meta_bytes = (size_t)N * NG * 4;
    uint8_t *area = blk + (isV ? code_bytes + meta_bytes : 0);
    uint32_t *codes_w = reinterpret_cast<uint32_t *>(area);
    uint32_t *meta_w = reinterpret_cast<uint32_t *>(area + code_bytes);
    const float qmax = (float)((1 << bits) - 1);

    for (int row = rsub; row < N; row += kPackThreads / 16) {
        const uint4 xv = *reinterpret_cast<const uint4 *>(src + (int64_t)row * a.stride_s + lane16 * 8);
        const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; e++) x[e] = half_bits_to_float((xw[e >> 1] >> (16 * (e & 1))) & 0xffffu);
        float mn = x[0], mx = x[0];
#pragma unroll
        for (int e = 1; e < 8; e++) { mn = fminf(mn, x[e]); mx = fmaxf(mx, x[e]); }
        mn = group_min<LPG>(mn);
        mx = group_max<LPG>(mx);
        if (mn == 0.0f) mn = 0.0f;                    // -0 is stored as +0
        if (mx == 0.0f) mx = 0.0f;
        const float R = __fsub_rn(mx, mn);
        const float s32 = __fdiv_rn(R, qmax);
        uint32_t s16 = float_to_half_bits(s32);
        if (half_bits_to_float(s16) < s32) s16 += 1;  // the scale is rounded up
        if (s16 == 0) s16 = 0x3C00u;                  // constant group: scale 1
        const float inv = __fdiv_rn(1.0f, half_bits_to_float(s16));
        uint32_t code[8];
#pragma unroll
        for (int e = 0; e < 8; e++) {
            float t = rintf(__fmul_rn(__fsub_rn(x[e], mn), inv));
            t = fminf(fmaxf(t, 0.0f), qmax);
            code[e] = (uint32_t)t;
        }
        if ((lane16 % LPG) == 0) meta_w[row * NG + lane16 / LPG] = s16 | (float_to_half_bits(mn) << 16);

        if (isV) {
            uint2 pk;
            pk.x = code[0] | code[1] << 8 | code[2] << 16 | code[3] << 24;
            pk.y = code[4] | code[5] << 8 | code[6] << 16 | code[7] << 24;
            *reinterpret_cast<uint2 *>(vcodes + row * kD + lane16 * 8) = pk;
        } else if (bits == 2) {                       // 16 dims per word: two lanes per word
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 8; e++) w |= code[e] << code_shift(e, 2);
            if (lane16 & 1) w <<= 8;                  // in-word indices 8..15
            w |= dpp_u<DPP_XOR1>(w);
            if (!(lane16 & 1)) codes_w[row * 8 + (lane16 >> 1)] = w;
        } else if (bits == 4) {                       // 8 dims per word: one lane per word
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 8; e++) w |= code[e] << code_shift(e, 4);
            codes_w[row * 16 + lane16] = w;
        } else {                                      // 8 bits, 4 dims per word: two words per lane
            uint2 w;
            w.x = code[0] | code[2] << 8 | code[1] << 16 | code[3] << 24;
            w.y = code[4] | code[6] << 8 | code[5] << 16 | code[7] << 24;
            *reinterpret_cast<uint2 *>(codes_w + row * 32 + lane16 * 2) = w;
        }
    }
    if (!isV) return;

    __syncthreads();
    // V: dimension-major 1-KiB tiles of 64 slots x 4 words.  A slot holds TQ = max(TW, 8) consecutive
    // tokens (TW = 32/bits per word, WD = TQ/TW words) of CPK = 4/WD dimensions that lie 16 apart;
    // slot 16*qd + j of tile cg of a block of 4*TQ tokens: dims 16*(cg*CPK + n/WD) + j, token slice qd.
    const int TW = 32 / bits, TQ = TW > 8 ? TW : 8, WD = TQ / TW, CPK = 4 / WD, NCG = kD / (16 * CPK);
    const int n_words = N * kD * bits / 32;
    for (int wv = tid; wv < n_words; wv += kPackThreads) {
        const int n = wv & 3, l = (wv >> 2) & 63, kib = wv >> 8;
        const int cg = kib % NCG, block = kib / NCG, qd = l >> 4, j = l & 15;
        const int d = 16 * (cg * CPK + n / WD) + j, t0 = block * 4 * TQ + qd * TQ + (n % WD) * TW;
        uint32_t w = 0;
        for (int e = 0; e < TW; e++) w |= (uint32_t)vcodes[(t0 + e) * kD + d] << code_shift(e, bits);
        codes_w[wv] = w;
    }
}

hipError_t launch_pack(const PackArgs &a, hipStream_t s) {
    if (a.n_chunks <= 0 || a.BH <= 0) return hipSuccess;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)a.n_chunks, (unsigned)a.BH, 2u);
    const size_t lds = (size_t)a.N * kD;
    if (a.G == 32) hipLaunchKernelGGL(pack_kernel<32>, grid, dim3(kPackThreads), lds, s, a);
    else           hipLaunchKernelGGL(pack_kernel<64>, grid, dim3(kPackThreads), lds, s, a);
    return hipGetLastError();
}

}  // namespace moqae
