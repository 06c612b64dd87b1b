// moqae_decode_attn: single-token decode attention over the mixed-precision packed cache with
// de-quantisation in registers and a binary32 online softmax ("Limitations" section of the
// paper: the quantised keys are de-quantised before they meet the query; softmax needs high
// precision).
//
// attn_split_kernel   grid (n_split, B*Hkv), 4 wavefronts per workgroup.  A workgroup owns a
//                     byte-balanced range of the row's chunks; its wavefronts take "units" of
//                     that range round-robin.  A unit is up to 4 KiB of K codes plus the
//                     matching 4 KiB of V codes (128 / 64 / 32 / 16 tokens at 2 / 4 / 8 / 16
//                     bits), loaded with one 16-byte load per lane per KiB.
//                     K: a lane holds 128/b consecutive codes of one token; V: a lane holds the
//                     codes of dims (2l, 2l+1) for the 64/b tokens of a tile.  Codes are never
//                     converted: masking a word leaves two codes in the mantissa fields of an
//                     fp16 pair (subnormal values code * 4^k * 2^-24, which v_dot2_f32_f16
//                     keeps), the power of four is folded into pre-scaled copies of q (K) or
//                     of the softmax weight (V), and the zero-points are factored out:
//                       q.k^   = sum_g scale_g * (sum_d code_d q_d) + zero_g * (sum_{d in g} q_d)
//                       sum p v^ = sum_t (p_t scale_tg) code_td  +  sum_t p_t zero_tg.
//                     Every wavefront writes one partial (m, l, o[D]).
// attn_merge_kernel   log-sum-exp merge of the partials of one query head, normalisation.
#include "moqae_dev.hpp"
#include "moqae_kernels.hpp"

namespace moqae {

constexpr int kAttnThreads = kAttnWaves * kWave;
constexpr float kTwo24 = 16777216.0f;
constexpr float kTwoM24 = 1.0f / 16777216.0f;

template <int BITS> struct BW {
    static constexpr int E = 128 / BITS;                 // codes in a 16-byte slot
    static constexpr int SPR = BITS;                     // slots (= lanes) per token row of 128 dims
    static constexpr int TT = 64 / BITS;                 // tokens per KiB of codes
    static constexpr int PS = E / 2;                     // fp16 pairs per slot
    static constexpr int PPW = BITS == 16 ? 1 : 16 / BITS;   // pairs per 32-bit word
    static constexpr int KD = BITS == 2 ? 5 : (BITS == 4 ? 2 : 1);  // pairs whose bits stay below the fp16 exponent
    static constexpr int SH = BITS == 2 ? 10 : 8;        // shift that brings the remaining pairs down
    static constexpr uint32_t MASK = BITS == 16 ? 0xffffffffu : ((1u << BITS) - 1u) * 0x00010001u;
    static constexpr int BI = BITS == 2 ? 0 : (BITS == 4 ? 1 : (BITS == 8 ? 2 : 3));
};

template <int G, int REP> struct alignas(16) AttnLds {
    static constexpr int NG = kD / G;
    uint32_t qtab[4][REP][64];                           // q as fp16 pairs, ordered and pre-scaled per bit-width
    float qpart[4][REP][16][2];                          // sum of q over a lane's dims (per group inside the slot)
    float sc[kAttnWaves][REP][128];                      // scores (log2 domain) / fp16-path weights of a unit
    uint16_t wl[kAttnWaves][REP][NG][128];               // fp16 softmax weight * V scale, pre-scaled per pair
    unsigned long long scan[kAttnThreads];
    int range[2];
};

// Orders this wavefront's LDS traffic between phases that exchange data across lanes.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int REP> struct WaveState {
    float m[REP], lsum[REP], z[REP], acc[REP][2];
};

// scale of the k-th pair of a word after masking: 2^(BITS*k') with k' counted from the shift
template <int BITS> __device__ __forceinline__ int pair_exp(int k) {
    return BITS * (k < BW<BITS>::KD ? k : k - BW<BITS>::KD);
}

// one 32-bit word of codes against PPW pre-scaled pairs
template <int BITS>
__device__ __forceinline__ float word_dot(uint32_t w, const uint32_t *pairs, float acc) {
    using B = BW<BITS>;
#pragma unroll
    for (int k = 0; k < B::KD; k++) acc = dot2(w & (B::MASK << (BITS * k)), pairs[k], acc);
    if constexpr (B::PPW > B::KD) {
        const uint32_t w2 = w >> B::SH;
#pragma unroll
        for (int k = B::KD; k < B::PPW; k++) acc = dot2(w2 & (B::MASK << (BITS * (k - B::KD))), pairs[k], acc);
    }
    return acc;
}

template <int REP>
__device__ __forceinline__ void rescale(WaveState<REP> &st, int r, float unit_max) {
    const float m_new = fmaxf(st.m[r], unit_max);
    const float alpha = fast_exp2(st.m[r] - m_new);       // first unit: exp2(-inf) = 0
    st.m[r] = m_new;
    st.lsum[r] *= alpha; st.z[r] *= alpha; st.acc[r][0] *= alpha; st.acc[r][1] *= alpha;
}

// ---- one unit of a quantised chunk -----------------------------------------------------------
template <int BITS, int G, int REP>
__device__ __forceinline__ void unit_quant(const uint8_t *__restrict__ kc, const uint32_t *__restrict__ km,
                                           const uint8_t *__restrict__ vc, const uint32_t *__restrict__ vm,
                                           int nsub, int lane, int wave, float scale_log2,
                                           AttnLds<G, REP> &L, WaveState<REP> &st) {
    using B = BW<BITS>;
    constexpr int NG = kD / G;
    constexpr int GS = (B::E > G) ? B::E / G : 1;        // groups inside one slot
    constexpr int MAXVM = (4 * B::TT * NG / 64) > 0 ? (4 * B::TT * NG / 64) : 1;
    const int part = lane % B::SPR, tok_l = lane / B::SPR;

    uint4 kbuf[4], vbuf[4];
    uint32_t kmeta[4][GS], vmeta[MAXVM];
    const int nvm = nsub * B::TT * NG / 64;
#pragma unroll
    for (int j = 0; j < 4; j++) if (j < nsub) {
        kbuf[j] = reinterpret_cast<const uint4 *>(kc)[64 * j + lane];
        const int g0 = (j * B::TT + tok_l) * NG + part * B::E / G;
#pragma unroll
        for (int gi = 0; gi < GS; gi++) kmeta[j][gi] = km[g0 + gi];
    }
#pragma unroll
    for (int j = 0; j < 4; j++) if (j < nsub) vbuf[j] = reinterpret_cast<const uint4 *>(vc)[64 * j + lane];
#pragma unroll
    for (int jj = 0; jj < MAXVM; jj++) if (jj < nvm) vmeta[jj] = vm[64 * jj + lane];

    // ---- scores
#pragma unroll
    for (int r = 0; r < REP; r++) {
        uint32_t qv[B::PS];
#pragma unroll
        for (int i = 0; i < B::PS; i += 4) {
            const uint4 t = *reinterpret_cast<const uint4 *>(&L.qtab[B::BI][r][part * B::PS + i]);
            qv[i] = t.x; qv[i + 1] = t.y; qv[i + 2] = t.z; qv[i + 3] = t.w;
        }
        float qp[GS];
#pragma unroll
        for (int gi = 0; gi < GS; gi++) qp[gi] = L.qpart[B::BI][r][part][gi];
        float s4[4], lmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            s4[j] = -INFINITY;
            if (j < nsub) {
                const uint32_t w[4] = {kbuf[j].x, kbuf[j].y, kbuf[j].z, kbuf[j].w};
                float ps = 0.0f;
#pragma unroll
                for (int gi = 0; gi < GS; gi++) {
                    float isum = 0.0f;
#pragma unroll
                    for (int wd = gi * (4 / GS); wd < (gi + 1) * (4 / GS); wd++)
                        isum = word_dot<BITS>(w[wd], &qv[wd * B::PPW], isum);
                    const float sK = half_bits_to_float(kmeta[j][gi] & 0xffffu) * kTwo24;
                    const float zK = half_bits_to_float(kmeta[j][gi] >> 16);
                    ps = fmaf(sK, isum, ps);
                    ps = fmaf(zK, qp[gi], ps);
                }
                ps = group_sum<B::SPR>(ps);
                s4[j] = ps * scale_log2;
                lmax = fmaxf(lmax, s4[j]);
            }
        }
        rescale(st, r, wave_max(lmax));
        if (part == 0) {
#pragma unroll
            for (int j = 0; j < 4; j++) if (j < nsub) L.sc[wave][r][j * B::TT + tok_l] = s4[j];
        }
    }

    wave_sync();
    // ---- softmax weights, one lane per V (token, group) meta word
    constexpr int n = 32 / BITS;
#pragma unroll
    for (int jj = 0; jj < MAXVM; jj++) if (jj < nvm) {
        const int idx = 64 * jj + lane, tv = idx / NG, g = idx % NG;
        const float sV = half_bits_to_float(vmeta[jj] & 0xffffu);
        const float zV = half_bits_to_float(vmeta[jj] >> 16);
        const int kk = (tv % n) >> 1;
        const int kp = BITS * (kk < B::KD ? kk : kk - B::KD);
        const float pre = sV * __builtin_bit_cast(float, (uint32_t)(127 - kp) << 23);
#pragma unroll
        for (int r = 0; r < REP; r++) {
            const float p = fast_exp2(L.sc[wave][r][tv] - st.m[r]);
            if (g == 0) st.lsum[r] += p;
            st.z[r] = fmaf(p, zV, st.z[r]);
            L.wl[wave][r][g][tv] = (uint16_t)float_to_half_bits(p * pre);
        }
    }

    wave_sync();
    // ---- weighted value sum: lane owns dims (2*lane, 2*lane+1)
    const int gl = (2 * lane) / G;
#pragma unroll
    for (int j = 0; j < 4; j++) if (j < nsub) {
        const uint32_t w[4] = {vbuf[j].x, vbuf[j].y, vbuf[j].z, vbuf[j].w};
#pragma unroll
        for (int r = 0; r < REP; r++) {
            uint32_t wp[2 * B::PPW];
#pragma unroll
            for (int i = 0; i < 2 * B::PPW; i += 4) {
                const uint4 t = *reinterpret_cast<const uint4 *>(&L.wl[wave][r][gl][j * B::TT + 2 * i]);
                wp[i] = t.x; wp[i + 1] = t.y; wp[i + 2] = t.z; wp[i + 3] = t.w;
            }
#pragma unroll
            for (int wd = 0; wd < 4; wd++)
                st.acc[r][wd >> 1] = word_dot<BITS>(w[wd], &wp[(wd & 1) * B::PPW], st.acc[r][wd >> 1]);
        }
    }
    wave_sync();
}

// ---- one unit of raw fp16 rows (16-bit chunks and the FP16 residual) -----------------------
template <int G, int REP>
__device__ __forceinline__ void unit_fp16(const uint8_t *__restrict__ krows, const uint8_t *__restrict__ vrows,
                                          int nsub, int nvalid, int lane, int wave, float scale_log2,
                                          AttnLds<G, REP> &L, WaveState<REP> &st) {
    const int part = lane & 15, tok_l = lane >> 4;
    const int ntok = 4 * nsub;
    uint4 kbuf[4];
    uint32_t vv[16];
#pragma unroll
    for (int j = 0; j < 4; j++) if (j < nsub) kbuf[j] = reinterpret_cast<const uint4 *>(krows)[64 * j + lane];
#pragma unroll
    for (int t = 0; t < 16; t++) if (t < ntok) vv[t] = reinterpret_cast<const uint32_t *>(vrows)[64 * t + lane];

#pragma unroll
    for (int r = 0; r < REP; r++) {
        const uint4 qv = *reinterpret_cast<const uint4 *>(&L.qtab[3][r][part * 4]);
        float s4[4], lmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            s4[j] = -INFINITY;
            if (j < nsub) {
                float ps = dot2(kbuf[j].x, qv.x, 0.0f);
                ps = dot2(kbuf[j].y, qv.y, ps);
                ps = dot2(kbuf[j].z, qv.z, ps);
                ps = dot2(kbuf[j].w, qv.w, ps);
                ps = group_sum<16>(ps);
                s4[j] = (4 * j + tok_l < nvalid) ? ps * scale_log2 : -INFINITY;
                lmax = fmaxf(lmax, s4[j]);
            }
        }
        rescale(st, r, wave_max(lmax));
        if (part == 0) {
#pragma unroll
            for (int j = 0; j < 4; j++) if (j < nsub) L.sc[wave][r][4 * j + tok_l] = s4[j];
        }
    }
    wave_sync();
#pragma unroll
    for (int r = 0; r < REP; r++) if (lane < ntok) {
        const float p = fast_exp2(L.sc[wave][r][lane] - st.m[r]);   // masked rows: exp2(-inf) = 0
        st.lsum[r] += p;
        L.sc[wave][r][lane] = p * kTwoM24;                           // accumulators carry a factor 2^-24
    }
    wave_sync();
#pragma unroll
    for (int t = 0; t < 16; t++) if (t < ntok && t < nvalid) {
        const float v0 = half_bits_to_float(vv[t] & 0xffffu), v1 = half_bits_to_float(vv[t] >> 16);
#pragma unroll
        for (int r = 0; r < REP; r++) {
            const float p = L.sc[wave][r][t];
            st.acc[r][0] = fmaf(p, v0, st.acc[r][0]);
            st.acc[r][1] = fmaf(p, v1, st.acc[r][1]);
        }
    }
    wave_sync();
}

template <int G, int REP>
__global__ __launch_bounds__(kAttnThreads) void attn_split_kernel(AttnArgs a) {
    __shared__ AttnLds<G, REP> L;
    constexpr int NG = kD / G;
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = (int)blockIdx.x, u = (int)blockIdx.y;
    const int N = a.N, C = a.n_chunks;
    const uint8_t *erow = a.expert + (int64_t)u * a.desc_stride;
    const uint64_t *orow = a.chunk_off + (int64_t)u * a.desc_stride;

    auto bits_of = [&](int e) {
        int b = 0;
#pragma unroll
        for (int k = 0; k < 8; k++) b = (e == k) ? a.bits_of[k] : b;
        return b;
    };

    // ---- byte-balanced chunk range of this split: chunk c belongs to the split that contains
    //      the byte position where its block starts in the row's concatenated blocks
    {
        const int per = (C + kAttnThreads - 1) / kAttnThreads;
        const int i0 = min(C, per * tid), i1 = min(C, i0 + per);
        unsigned long long local = 0;
        for (int c = i0; c < i1; c++) local += block_bytes(N, G, bits_of(erow[c]));
        L.scan[tid] = local;
        if (tid == 0) { L.range[0] = C; L.range[1] = C; }
        __syncthreads();
        for (int off = 1; off < kAttnThreads; off <<= 1) {
            unsigned long long v = tid >= off ? L.scan[tid - off] : 0;
            __syncthreads();
            L.scan[tid] += v;
            __syncthreads();
        }
        const unsigned long long total = L.scan[kAttnThreads - 1];
        const unsigned long long lo = total / a.n_split * split + total % a.n_split * split / a.n_split;
        const unsigned long long hi = (split == a.n_split - 1) ? total
                                    : total / a.n_split * (split + 1) + total % a.n_split * (split + 1) / a.n_split;
        unsigned long long pos = L.scan[tid] - local;
        int f0 = C, f1 = C;
        for (int c = i0; c < i1; c++) {
            if (f0 == C && pos >= lo) f0 = c;
            if (f1 == C && pos >= hi) f1 = c;
            pos += block_bytes(N, G, bits_of(erow[c]));
        }
        if (f0 < C) atomicMin(&L.range[0], f0);
        if (f1 < C) atomicMin(&L.range[1], f1);
    }

    // ---- q tables: per bit-width the pairs in the order the unpacking produces them
    {
        const int b = u / a.Hkv, h = u % a.Hkv;
        const uint16_t *qrow = a.q + ((int64_t)b * a.Hkv * REP + (int64_t)h * REP) * kD;
        for (int i = tid; i < 4 * REP * 64; i += kAttnThreads) {
            const int bi = i / (REP * 64), r = (i / 64) % REP, ent = i % 64;
            const int BITSv = 2 << bi;
            const int ps = 64 / BITSv, ppw = bi == 3 ? 1 : 16 / BITSv, kd = bi == 0 ? 5 : (bi == 1 ? 2 : 1);
            const int part = ent / ps, ii = ent % ps, j = ii / ppw, k = ii % ppw;
            const int d0 = part * (128 / BITSv) + j * 2 * ppw + 2 * k;
            const int kp = bi == 3 ? 0 : BITSv * (k < kd ? k : k - kd);
            const float f = __builtin_bit_cast(float, (uint32_t)(127 - kp) << 23);
            const uint32_t lo16 = float_to_half_bits(half_bits_to_float(qrow[r * kD + d0]) * f);
            const uint32_t hi16 = float_to_half_bits(half_bits_to_float(qrow[r * kD + d0 + 1]) * f);
            L.qtab[bi][r][ent] = lo16 | (hi16 << 16);
        }
        for (int i = tid; i < 4 * REP * 16 * 2; i += kAttnThreads) {
            const int bi = i / (REP * 32), r = (i / 32) % REP, part = (i / 2) % 16, gi = i % 2;
            const int BITSv = 2 << bi, E = 128 / BITSv;
            float s = 0.0f;
            if (part < BITSv) {
                const int gs = E > G ? E / G : 1;
                if (gi < gs) {
                    const int len = E / gs, d0 = part * E + gi * len;
                    for (int d = 0; d < len; d++) s += half_bits_to_float(qrow[r * kD + d0 + d]);
                }
            }
            L.qpart[bi][r][part][gi] = s;
        }
    }
    __syncthreads();
    const int c0 = L.range[0], c1 = L.range[1];

    WaveState<REP> st;
#pragma unroll
    for (int r = 0; r < REP; r++) { st.m[r] = -INFINITY; st.lsum[r] = 0.0f; st.z[r] = 0.0f; st.acc[r][0] = 0.0f; st.acc[r][1] = 0.0f; }

    int ucount = 0;
    for (int cbase = c0; cbase < c1; cbase += 64) {
        const int nb = min(64, c1 - cbase);
        int my_bits = 0; unsigned long long my_off = 0;
        if (lane < nb) { my_bits = bits_of(erow[cbase + lane]); my_off = orow[cbase + lane]; }
        for (int i = 0; i < nb; i++) {
            const int bits = __builtin_amdgcn_readlane(my_bits, i);
            const unsigned long long off = (unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)my_off, i)
                                         | ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(my_off >> 32), i) << 32);
            const uint8_t *blk = a.arena + off;
            const int TT = 64 / bits;
            const int nu = (N + 4 * TT - 1) / (4 * TT);         // units of up to 4 KiB of codes
            for (int s = 0; s < nu; s++) {
                if (((ucount + s) & (kAttnWaves - 1)) != wave) continue;
                const int t0 = s * 4 * TT;
                const int nsub = min(4, (N - t0) / TT);          // the last unit of a chunk may be short
                const int ut = nsub * TT;
                if (bits == 16) {
                    unit_fp16<G, REP>(blk + (size_t)t0 * 256, blk + (size_t)N * 256 + (size_t)t0 * 256,
                                      nsub, ut, lane, wave, a.scale_log2, L, st);
                } else {
                    const size_t cb = (size_t)N * 16 * bits, mb = (size_t)N * NG * 4;
                    const uint8_t *kc = blk + (size_t)t0 * 16 * bits;
                    const uint32_t *km = reinterpret_cast<const uint32_t *>(blk + cb) + t0 * NG;
                    const uint8_t *vc = blk + cb + mb + (size_t)t0 * 16 * bits;
                    const uint32_t *vm = reinterpret_cast<const uint32_t *>(blk + 2 * cb + mb) + t0 * NG;
                    if (bits == 2)      unit_quant<2, G, REP>(kc, km, vc, vm, nsub, lane, wave, a.scale_log2, L, st);
                    else if (bits == 4) unit_quant<4, G, REP>(kc, km, vc, vm, nsub, lane, wave, a.scale_log2, L, st);
                    else                unit_quant<8, G, REP>(kc, km, vc, vm, nsub, lane, wave, a.scale_log2, L, st);
                }
            }
            ucount += nu;
        }
    }
    if (split == a.n_split - 1 && a.n_tail > 0) {          // FP16 residual rows
        const int nut = (a.n_tail + 15) / 16;
        for (int s = 0; s < nut; s++) {
            if (((ucount + s) & (kAttnWaves - 1)) != wave) continue;
            const size_t rowb = ((size_t)u * N + (size_t)16 * s) * 256;
            unit_fp16<G, REP>(reinterpret_cast<const uint8_t *>(a.K_tail) + rowb,
                              reinterpret_cast<const uint8_t *>(a.V_tail) + rowb,
                              4, min(16, a.n_tail - 16 * s), lane, wave, a.scale_log2, L, st);
        }
    }

    // ---- the wavefront's partial: o[d] = acc[d] * 2^24 + sum_t p_t zero_{t,g(d)}, plus (m, l)
    const int P = a.n_split * kAttnWaves;
#pragma unroll
    for (int r = 0; r < REP; r++) {
        float lt = st.lsum[r], zt = st.z[r];
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) lt += __shfl_xor(lt, o);
#pragma unroll
        for (int o = 32; o >= NG; o >>= 1) zt += __shfl_xor(zt, o);   // lanes with equal lane % NG
        const float zg = __shfl(zt, (2 * lane) / G);
        float *dst = a.part + (((int64_t)u * REP + r) * P + (int64_t)split * kAttnWaves + wave) * (kD + 2);
        float2 o2; o2.x = fmaf(st.acc[r][0], kTwo24, zg); o2.y = fmaf(st.acc[r][1], kTwo24, zg);
        *reinterpret_cast<float2 *>(dst + 2 * lane) = o2;
        if (lane == 0) { dst[kD] = st.m[r]; dst[kD + 1] = lt; }
    }
}

// out[b, hq, :] = sum_p o_p 2^(m_p - M) / sum_p l_p 2^(m_p - M)
__global__ __launch_bounds__(kD) void attn_merge_kernel(const float *__restrict__ part, float *__restrict__ out, int P) {
    const int row = (int)blockIdx.x, d = (int)threadIdx.x;
    const float *p0 = part + (int64_t)row * P * (kD + 2);
    float M = -INFINITY;
    for (int p = 0; p < P; p++) M = fmaxf(M, p0[p * (kD + 2) + kD]);
    float num = 0.0f, den = 0.0f;
    for (int p = 0; p < P; p++) {
        const float *pp = p0 + p * (kD + 2);
        const float f = fast_exp2(pp[kD] - M);               // empty partial: m = -inf -> 0
        num = fmaf(pp[d], f, num);
        den = fmaf(pp[kD + 1], f, den);
    }
    out[(int64_t)row * kD + d] = num / den;
}

template <int G, int REP>
static hipError_t launch_gr(const AttnArgs &a, hipStream_t s) {
    hipLaunchKernelGGL((attn_split_kernel<G, REP>), dim3((unsigned)a.n_split, (unsigned)a.BH), dim3(kAttnThreads), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attn_merge_kernel, dim3((unsigned)(a.BH * a.rep)), dim3(kD), 0, s,
                       (const float *)a.part, a.out, a.n_split * kAttnWaves);
    return hipGetLastError();
}

hipError_t launch_attn(const AttnArgs &a, hipStream_t s) {
#define MOQAE_CASE(GV, RV) if (a.G == GV && a.rep == RV) return launch_gr<GV, RV>(a, s);
    MOQAE_CASE(64, 1) MOQAE_CASE(64, 2) MOQAE_CASE(64, 4) MOQAE_CASE(64, 8)
    MOQAE_CASE(32, 1) MOQAE_CASE(32, 2) MOQAE_CASE(32, 4) MOQAE_CASE(32, 8)
#undef MOQAE_CASE
    return hipErrorInvalidValue;
}

}  // namespace moqae
