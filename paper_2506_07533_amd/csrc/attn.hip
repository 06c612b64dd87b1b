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

// A unit: up to 4 KiB of K codes (nsub KiB) with the matching V codes; wave-uniform.
struct Unit {
    int bits, nsub, nvalid;                              // nvalid: valid rows of an fp16 unit
    const uint8_t *kc, *vc;
    const uint32_t *km, *vm;
};

template <int G> struct KRegs {
    static constexpr int GSMAX = (G == 32) ? 2 : 1;      // a 2-bit slot of 64 codes spans two groups of 32
    uint4 c[4];
    uint32_t m[4][GSMAX];
};

// Loads the K side of a unit whatever its bit-width: lane l takes the 16-byte slot 64*j + l of
// each KiB and the meta word(s) of the (token, group) that slot belongs to.  Branch-free: a
// short unit (nsub < 4) re-reads its last KiB and an fp16 unit reads four words of its own rows
// in place of the meta words it does not have; both are ignored by the consumer.
template <int G>
__device__ __forceinline__ void load_k(const Unit &u, int lane, KRegs<G> &k) {
    constexpr int NG = kD / G;
    const int lg = u.bits == 2 ? 1 : (u.bits == 4 ? 2 : 3);          // log2(lanes per token row)
    const int TT = 64 >> lg, E = 128 >> lg;
    const int tok_l = lane >> lg, part = lane & ((1 << lg) - 1);
    const int g_in_row = part * E / G;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const int jc = min(j, u.nsub - 1);
        k.c[j] = reinterpret_cast<const uint4 *>(u.kc)[64 * jc + lane];
        const int g0 = (jc * TT + tok_l) * NG + g_in_row;
        k.m[j][0] = u.km[g0];
        if constexpr (KRegs<G>::GSMAX == 2) k.m[j][1] = u.km[g0 + (E > G ? 1 : 0)];
    }
}

// ---- one unit of a quantised chunk -----------------------------------------------------------
template <int BITS, int G, int REP, class Prefetch>
__device__ __forceinline__ void unit_quant(const Unit &u, KRegs<G> &k, Prefetch &&prefetch,
                                           int lane, int wave, float scale_log2,
                                           AttnLds<G, REP> &L, WaveState<REP> &st) {
    using B = BW<BITS>;
    constexpr int NG = kD / G;
    constexpr int GS = (B::E > G) ? B::E / G : 1;        // groups inside one slot
    constexpr int MAXVM = (4 * B::TT * NG / 64) > 0 ? (4 * B::TT * NG / 64) : 1;
    const int part = lane % B::SPR, tok_l = lane / B::SPR;
    const int nsub = u.nsub;

    uint4 vbuf[4];
    uint32_t vmeta[MAXVM];
    const int nvm = nsub * B::TT * NG / 64;              // >= 1
#pragma unroll
    for (int j = 0; j < 4; j++) vbuf[j] = reinterpret_cast<const uint4 *>(u.vc)[64 * min(j, nsub - 1) + lane];
#pragma unroll
    for (int jj = 0; jj < MAXVM; jj++) vmeta[jj] = u.vm[64 * min(jj, nvm - 1) + lane];

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
            const uint32_t w[4] = {k.c[j].x, k.c[j].y, k.c[j].z, k.c[j].w};
            float ps = 0.0f;
#pragma unroll
            for (int gi = 0; gi < GS; gi++) {
                float isum = 0.0f;
#pragma unroll
                for (int wd = gi * (4 / GS); wd < (gi + 1) * (4 / GS); wd++)
                    isum = word_dot<BITS>(w[wd], &qv[wd * B::PPW], isum);
                const float sK = half_bits_to_float(k.m[j][gi] & 0xffffu) * kTwo24;
                const float zK = half_bits_to_float(k.m[j][gi] >> 16);
                ps = fmaf(sK, isum, ps);
                ps = fmaf(zK, qp[gi], ps);
            }
            ps = group_sum<B::SPR>(ps);
            s4[j] = (j < nsub) ? ps * scale_log2 : -INFINITY;     // KiB past a short unit: ignored
            lmax = fmaxf(lmax, s4[j]);
        }
        rescale(st, r, wave_max(lmax));
        if (part == 0) {
#pragma unroll
            for (int j = 0; j < 4; j++) L.sc[wave][r][j * B::TT + tok_l] = s4[j];
        }
    }
    prefetch();                                          // K side of the wavefront's next unit

    wave_sync();
    // ---- softmax weights, one lane per V (token, group) meta word
    constexpr int n = 32 / BITS;
#pragma unroll
    for (int jj = 0; jj < MAXVM; jj++) {
        const int idx = 64 * jj + lane, tv = idx / NG, g = idx % NG;
        const float sV = half_bits_to_float(vmeta[jj] & 0xffffu);
        const float zV = half_bits_to_float(vmeta[jj] >> 16);
        const int kk = (tv % n) >> 1;
        const int kp = BITS * (kk < B::KD ? kk : kk - B::KD);
        const float pre = sV * __builtin_bit_cast(float, (uint32_t)(127 - kp) << 23);
#pragma unroll
        for (int r = 0; r < REP; r++) {
            const float p = fast_exp2(L.sc[wave][r][tv] - st.m[r]);   // tokens past a short unit: score -inf, p = 0
            if (g == 0) st.lsum[r] += p;
            st.z[r] = fmaf(p, zV, st.z[r]);
            L.wl[wave][r][g][tv] = (uint16_t)float_to_half_bits(p * pre);
        }
    }

    wave_sync();
    // ---- weighted value sum: lane owns dims (2*lane, 2*lane+1)
    const int gl = (2 * lane) / G;
#pragma unroll
    for (int j = 0; j < 4; j++) {
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
template <int G, int REP, class Prefetch>
__device__ __forceinline__ void unit_fp16(const Unit &u, KRegs<G> &k, Prefetch &&prefetch,
                                          int lane, int wave, float scale_log2,
                                          AttnLds<G, REP> &L, WaveState<REP> &st) {
    const int part = lane & 15, tok_l = lane >> 4;
    const int nvalid = u.nvalid;                          // an fp16 unit always spans 16 rows
    uint32_t vv[16];
#pragma unroll
    for (int t = 0; t < 16; t++) vv[t] = reinterpret_cast<const uint32_t *>(u.vc)[64 * t + lane];

#pragma unroll
    for (int r = 0; r < REP; r++) {
        const uint4 qv = *reinterpret_cast<const uint4 *>(&L.qtab[3][r][part * 4]);
        float s4[4], lmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            float ps = dot2(k.c[j].x, qv.x, 0.0f);
            ps = dot2(k.c[j].y, qv.y, ps);
            ps = dot2(k.c[j].z, qv.z, ps);
            ps = dot2(k.c[j].w, qv.w, ps);
            ps = group_sum<16>(ps);
            s4[j] = (4 * j + tok_l < nvalid) ? ps * scale_log2 : -INFINITY;
            lmax = fmaxf(lmax, s4[j]);
        }
        rescale(st, r, wave_max(lmax));
        if (part == 0) {
#pragma unroll
            for (int j = 0; j < 4; j++) L.sc[wave][r][4 * j + tok_l] = s4[j];
        }
    }
    prefetch();

    wave_sync();
#pragma unroll
    for (int r = 0; r < REP; r++) {
        const float p = fast_exp2(L.sc[wave][r][lane & 15] - st.m[r]);   // masked rows: exp2(-inf) = 0
        if (lane < 16) {
            st.lsum[r] += p;
            L.sc[wave][r][lane] = p * kTwoM24;                        // accumulators carry a factor 2^-24
        }
    }
    wave_sync();
#pragma unroll
    for (int t = 0; t < 16; t++) {
        // rows past nvalid may hold anything (NaN, Inf): select, do not multiply by zero
        const float v0 = (t < nvalid) ? half_bits_to_float(vv[t] & 0xffffu) : 0.0f;
        const float v1 = (t < nvalid) ? half_bits_to_float(vv[t] >> 16) : 0.0f;
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
__global__ __launch_bounds__(kAttnThreads, (REP == 1 ? 4 : 2)) void attn_split_kernel(AttnArgs a) {
    __shared__ AttnLds<G, REP> L;
    constexpr int NG = kD / G;
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);           // wave-uniform, kept scalar
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
        unsigned long long incl = local;                   // inclusive scan inside the wavefront
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long v = __shfl_up(incl, o);
            if (lane >= o) incl += v;
        }
        if (lane == 63) L.scan[wave] = incl;
        if (tid == 0) { L.range[0] = C; L.range[1] = C; }
        __syncthreads();
        unsigned long long base = 0, total = 0;
#pragma unroll
        for (int wv = 0; wv < kAttnWaves; wv++) { if (wv < wave) base += L.scan[wv]; total += L.scan[wv]; }
        const unsigned long long lo = total / a.n_split * split + total % a.n_split * split / a.n_split;
        const unsigned long long hi = (split == a.n_split - 1) ? total
                                    : total / a.n_split * (split + 1) + total % a.n_split * (split + 1) / a.n_split;
        unsigned long long pos = base + incl - local;
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
    const int c0 = __builtin_amdgcn_readfirstlane(L.range[0]), c1 = __builtin_amdgcn_readfirstlane(L.range[1]);

    WaveState<REP> st;
#pragma unroll
    for (int r = 0; r < REP; r++) { st.m[r] = -INFINITY; st.lsum[r] = 0.0f; st.z[r] = 0.0f; st.acc[r][0] = 0.0f; st.acc[r][1] = 0.0f; }

    // ---- this wavefront's units: every 4th unit of the range (and of the FP16 residual, which
    //      the last split takes), enumerated chunk by chunk
    const bool has_tail = split == a.n_split - 1 && a.n_tail > 0;
    int ci = c0, cbase = c0, nbatch = 0, s_next = 0, ucount = 0, my_bits = 0;
    unsigned long long my_off = 0;
    bool in_tail = false;
    auto next_unit = [&](Unit &un) -> bool {
        for (;;) {
            if (!in_tail) {
                if (ci >= c1) {
                    if (!has_tail) return false;
                    in_tail = true; s_next = 0;
                    continue;
                }
                if (ci >= cbase + nbatch) {                 // next batch of 64 chunk descriptors
                    cbase = ci; nbatch = min(64, c1 - cbase);
                    my_bits = 0; my_off = 0;
                    if (lane < nbatch) { my_bits = bits_of(erow[cbase + lane]); my_off = orow[cbase + lane]; }
                }
                const int i = ci - cbase;
                const int bits = __builtin_amdgcn_readlane(my_bits, i);
                const int TT = 64 / bits;
                const int nu = (N + 4 * TT - 1) / (4 * TT);
                const int s = s_next + ((wave - (ucount + s_next)) & (kAttnWaves - 1));
                if (s < nu) {
                    const unsigned long long off =
                        (unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)my_off, i) |
                        ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(my_off >> 32), i) << 32);
                    const uint8_t *blk = a.arena + off;
                    const int t0 = s * 4 * TT;
                    un.bits = bits; un.nsub = min(4, (N - t0) / TT); un.nvalid = un.nsub * TT;
                    if (bits == 16) {
                        un.kc = blk + (size_t)t0 * 256; un.vc = blk + (size_t)N * 256 + (size_t)t0 * 256;
                        un.km = reinterpret_cast<const uint32_t *>(un.kc); un.vm = un.km;   // no meta: see load_k
                    } else {
                        const size_t cb = (size_t)N * 16 * bits, mb = (size_t)N * NG * 4;
                        un.kc = blk + (size_t)t0 * 16 * bits;
                        un.km = reinterpret_cast<const uint32_t *>(blk + cb) + t0 * NG;
                        un.vc = blk + cb + mb + (size_t)t0 * 16 * bits;
                        un.vm = reinterpret_cast<const uint32_t *>(blk + 2 * cb + mb) + t0 * NG;
                    }
                    s_next = s + 1;
                    return true;
                }
                ucount += nu; ci++; s_next = 0;
            } else {
                const int nu = (a.n_tail + 15) / 16;
                const int s = s_next + ((wave - (ucount + s_next)) & (kAttnWaves - 1));
                if (s >= nu) return false;
                const size_t rowb = ((size_t)u * N + (size_t)16 * s) * 256;
                un.bits = 16; un.nsub = 4; un.nvalid = min(16, a.n_tail - 16 * s);
                un.kc = reinterpret_cast<const uint8_t *>(a.K_tail) + rowb;
                un.vc = reinterpret_cast<const uint8_t *>(a.V_tail) + rowb;
                un.km = reinterpret_cast<const uint32_t *>(un.kc); un.vm = un.km;
                s_next = s + 1;
                return true;
            }
        }
    };

    Unit cur, nxt;
    KRegs<G> kr;
    bool have = next_unit(cur);
    if (have) load_k<G>(cur, lane, kr);
    while (have) {
        const bool have_next = next_unit(nxt);
        const Unit &pf = have_next ? nxt : cur;          // nothing left: re-read the current unit (ignored)
        auto prefetch = [&]() { load_k<G>(pf, lane, kr); };
        if (cur.bits == 2)      unit_quant<2, G, REP>(cur, kr, prefetch, lane, wave, a.scale_log2, L, st);
        else if (cur.bits == 4) unit_quant<4, G, REP>(cur, kr, prefetch, lane, wave, a.scale_log2, L, st);
        else if (cur.bits == 8) unit_quant<8, G, REP>(cur, kr, prefetch, lane, wave, a.scale_log2, L, st);
        else                    unit_fp16<G, REP>(cur, kr, prefetch, lane, wave, a.scale_log2, L, st);
        cur = nxt; have = have_next;
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

// out[b, hq, :] = sum_p o_p 2^(m_p - M) / sum_p l_p 2^(m_p - M) over the P partials of the row.
constexpr int kMergeGroups = 4;
__global__ __launch_bounds__(kD *kMergeGroups) void attn_merge_kernel(const float *__restrict__ part,
                                                                       float *__restrict__ out, int P) {
    __shared__ float red[kD * kMergeGroups];
    __shared__ float numl[kMergeGroups][kD];
    __shared__ float denl[kMergeGroups];
    const int row = (int)blockIdx.x, tid = (int)threadIdx.x, d = tid & (kD - 1), grp = tid >> 7;
    const float *p0 = part + (int64_t)row * P * (kD + 2);
    float mx = -INFINITY;
    for (int p = tid; p < P; p += kD * kMergeGroups) mx = fmaxf(mx, p0[(int64_t)p * (kD + 2) + kD]);
    red[tid] = mx;
    __syncthreads();
    for (int o = kD * kMergeGroups / 2; o >= 1; o >>= 1) {
        if (tid < o) red[tid] = fmaxf(red[tid], red[tid + o]);
        __syncthreads();
    }
    const float M = red[0];
    float num = 0.0f, den = 0.0f;
#pragma unroll 4
    for (int p = grp; p < P; p += kMergeGroups) {
        const float *pp = p0 + (int64_t)p * (kD + 2);
        const float f = fast_exp2(pp[kD] - M);               // empty partial: m = -inf -> 0
        num = fmaf(pp[d], f, num);
        den = fmaf(pp[kD + 1], f, den);
    }
    numl[grp][d] = num;
    if (d == 0) denl[grp] = den;
    __syncthreads();
    if (grp == 0) {
        float n = 0.0f, dn = 0.0f;
#pragma unroll
        for (int g = 0; g < kMergeGroups; g++) { n += numl[g][d]; dn += denl[g]; }
        out[(int64_t)row * kD + d] = n / dn;
    }
}

template <int G, int REP>
static int resident_wgs_per_cu() {
    static int cached = 0;
    if (cached == 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attn_split_kernel<G, REP>, kAttnThreads, 0) != hipSuccess || n < 1)
            n = 1;
        cached = n;
    }
    return cached;
}

template <int G, int REP>
static hipError_t launch_gr(const AttnArgs &a, hipStream_t s) {
    hipLaunchKernelGGL((attn_split_kernel<G, REP>), dim3((unsigned)a.n_split, (unsigned)a.BH), dim3(kAttnThreads), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attn_merge_kernel, dim3((unsigned)(a.BH * a.rep)), dim3(kD * kMergeGroups), 0, s,
                       (const float *)a.part, a.out, a.n_split * kAttnWaves);
    return hipGetLastError();
}

#define MOQAE_FOR_EACH_VARIANT(X) X(64, 1) X(64, 2) X(64, 4) X(64, 8) X(32, 1) X(32, 2) X(32, 4) X(32, 8)

int attn_resident_wgs_per_cu(int G, int rep) {
#define MOQAE_CASE(GV, RV) if (G == GV && rep == RV) return resident_wgs_per_cu<GV, RV>();
    MOQAE_FOR_EACH_VARIANT(MOQAE_CASE)
#undef MOQAE_CASE
    return 1;
}

hipError_t launch_attn(const AttnArgs &a, hipStream_t s) {
#define MOQAE_CASE(GV, RV) if (a.G == GV && a.rep == RV) return launch_gr<GV, RV>(a, s);
    MOQAE_FOR_EACH_VARIANT(MOQAE_CASE)
#undef MOQAE_CASE
    return hipErrorInvalidValue;
}

}  // namespace moqae
