// moqae_decode_attn: single-token decode attention over the mixed-precision packed cache with
// de-quantisation in registers and a binary32 online softmax ("Limitations" section of the
// paper: the quantised keys are de-quantised before they meet the query; softmax needs high
// precision).
//
// attn_prep_kernel    zeroes the ticket counters and counts the units of every (sequence, KV head) row.
// attn_split_kernel   one persistent workgroup per CU (8 wavefronts).  A workgroup owns an interval
//                     of the rows, balanced by units; inside a row its wavefronts draw tickets
//                     (one "unit" each) from counters shared by the workgroups of the row.  A unit is
//                     up to 4 KiB of K codes plus the matching 4 KiB of V codes (128 / 64 / 32 / 16
//                     tokens at 2 / 4 / 8 / 16 bits), loaded with one 16-byte load per lane per KiB.
//                     Codes are never converted one by one.  The zero-points are factored out,
//                       q.k^   = sum_g scale_g * (sum_d code_d q_d) + zero_g * (sum_{d in g} q_d)
//                       sum p v^ = sum_t (p_t scale_tg) code_td  +  sum_t p_t zero_tg,
//                     and the code sums run on the matrix cores:
//                     - one query head per KV head: byte-wise masks leave one code per byte and
//                       v_mfma_i32_16x16x64_i8 multiplies them with the base-128 digits of a
//                       fixed-point copy of q (scores) or of the softmax weights (values);
//                     - grouped queries: masking a word leaves two codes in the mantissa fields of an
//                       fp16 pair (subnormal values code * 4^k * 2^-24, which the matrix core keeps)
//                       and v_mfma_f32_16x16x32_f16 multiplies them with pre-scaled copies of q / of
//                       the weights, all heads of the group in one product;
//                     - raw fp16 rows (16-bit chunks, FP16 residual): v_dot2_f32_f16 / mixed FMAs.
//                     Every workgroup writes one partial (m, l, o[D]) per row it touched.
// attn_merge_kernel   log-sum-exp merge of the partials of one query head, normalisation.
#include <type_traits>
#include "moqae_dev.hpp"
#include "moqae_kernels.hpp"

namespace moqae {

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

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kDescCap = 1024;                            // chunks of a row segment (descriptors held in LDS)
constexpr int kUnitCap = 8192;                            // units of a row segment
constexpr int kCounterStride = 64;                        // uint32 slots between two ticket counters (256 bytes)
constexpr int kMaxWeightedRowsLds = 1024;                // == kMaxWeightedRows
constexpr int kMaxBatches = 64;                           // ticket batches a workgroup can be granted per row segment
constexpr uint32_t kRowSetupCost = 40u * 16u;             // a row's set-up in the cost unit of attn_prep_kernel (512 bytes of codes)

template <int G, int REP, int NWV> struct alignas(16) AttnLds {
    static constexpr int NG = kD / G;
    uint32_t qtab[REP][64];                              // q as fp16 pairs in the order of the raw fp16 rows
    // one query head per KV head: operands and constants of the integer matrix-core path (see iq_build_q)
    v4i qa[REP == 1 ? 8 : 1][64];
    v4i wa[REP == 1 ? NWV : 1][2][64];                   // per wavefront: weight digits of up to two token blocks
    uint32_t wpos[REP == 1 ? 3 : 1][8][64];
    alignas(16) float vf[REP < 4 ? NWV : 1][512];                  // raw fp16 units: the value sums of the four row groups on their way to the lanes that own the dims
    uint4 kx[REP == 1 ? NWV : 1][4 * 72];                // per wavefront: the K codes of a unit on their way to the lanes that use them
    alignas(16) float pcq[REP == 1 ? NWV : 1][4][kD];    // keys quantised per channel: q * scale of up to four token groups of a unit
    int iq[kD];
    int iqs16[8];
    float iqpart[3][8][2];
    float iqscale[4];
    float sc[NWV][REP][128];                             // scores (log2 domain) / fp16-path weights of a unit
    static constexpr int WLS = 136;                      // weight row stride in halfs: rows fall on different banks
    alignas(16) uint16_t wl[NWV][REP][NG][WLS];                     // fp16 softmax weight * V scale, pre-scaled per pair
    uint16_t zrow[WLS];                                  // zeros: the weight row of the unused tile rows
    float qsumg[REP][NG];                                // sum of q over a group, times 2^-24
    v4u qmc[REP > 1 ? 3 : 1][4][REP > 1 ? 64 : 1];       // grouped queries: score operands A per (bit-width, pass, lane)
    float comb[NWV][REP][kD + 2];                        // per-wavefront (o, m, l) at the end of a row segment
    uint32_t qraw[REP * 64];                             // the row's queries as loaded (fp16 pairs)
    unsigned long long desc[kDescCap];                   // chunk descriptors of the current pass: offset | expert
    // ticket queue of the workgroup: local tickets [0, limit) are granted; batch i maps local
    // tickets from bl[i] on to the row's tickets from bg[i] on
    uint16_t ustart[kDescCap];                           // first unit of every chunk of the segment
    uint16_t inv[kUnitCap];                              // unit -> chunk of the segment
    uint32_t wscan[NWV];
    uint32_t U[kMaxWeightedRowsLds + 1], r0;            // prefix sums of the rows' units
    uint32_t next, limit, done, fetching, g_seen, nb;
    uint32_t bl[kMaxBatches], bg[kMaxBatches];
};

// Inclusive prefix sum over the 64 lanes, on the vector ALU (row shifts, then the row totals handed on).
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x) {
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xF, 0xF, false);   // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xF, 0xF, false);   // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xF, 0xF, false);   // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xF, 0xF, false);   // row_shr:8
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, DPP_BCAST15, 0xA, 0xF, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, DPP_BCAST31, 0xC, 0xF, false);
    return x;
}

// Orders this wavefront's LDS traffic between phases that exchange data across lanes.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int REP> struct WaveState {
    float m[REP], lsum[REP], z[REP];
    float acc[REP][2];                                   // raw fp16 rows: dims (2l, 2l+1), in units of 2^-24
    float accq[REP][8];                                  // quantised V, one head per KV head: dims 16*ct + l%16, this lane's token slices only
    v4f accA[8];                                         // quantised V, grouped queries: matrix-core tile ct, rows 4*(l/16)..+3
};

// scale of the k-th pair of a word after masking: 2^(BITS*k') with k' counted from the shift
template <int BITS> __device__ __forceinline__ int pair_exp(int k) {
    return BITS * (k < BW<BITS>::KD ? k : k - BW<BITS>::KD);
}

// New running maximum of head r: every accumulator of the head is scaled by 2^(old - new).
template <int G, int REP>
__device__ __forceinline__ void rescale(WaveState<REP> &st, int r, float unit_max, int lane) {
    const float m_new = fmaxf(st.m[r], unit_max);
    const float alpha = (m_new == -INFINITY) ? 1.0f : fast_exp2(st.m[r] - m_new);   // first unit: exp2(-inf) = 0; nothing seen yet: unchanged
    st.m[r] = m_new;
    st.lsum[r] *= alpha; st.z[r] *= alpha; st.acc[r][0] *= alpha; st.acc[r][1] *= alpha;
    if constexpr (REP == 1) {
#pragma unroll
        for (int ct = 0; ct < 8; ct++) st.accq[r][ct] *= alpha;
    } else {
        if (alpha != 1.0f) {                              // wave-uniform; rare once the maximum has settled
            constexpr int NG = kD / G;
            const int qd = lane >> 4;
#pragma unroll
            for (int n = 0; n < 4; n++) {
                const float f = ((4 * qd + n) / NG == r) ? alpha : 1.0f;         // tile rows >= REP*NG hold zeros
#pragma unroll
                for (int ct = 0; ct < 8; ct++) st.accA[ct][n] *= f;
            }
        }
    }
}

// A unit: up to 4 KiB of K codes (nsub KiB) with the matching V codes.  All fields are
// wave-uniform and live in scalar registers; lgb = log2(bit-width) (1, 2, 3; 4 = raw fp16).
struct Unit {
    int lgb, nsub, nvalid;                               // nvalid: valid rows of an fp16 unit
    int tail_rows;                                       // residual units: valid residual rows from the unit's first row on (else huge)
    const uint8_t *kb, *vb;                              // bases: the chunk block (both), or the residual K and V rows of the row
    uint32_t kc, km, vc, vm;                             // byte offsets of the unit's K codes / K meta (from kb), V codes / V meta (from vb)
};

template <int G> struct KRegs {
    static constexpr int GSMAX = 2;                      // a 2-bit slot of 64 codes spans two groups of 32; per-channel keys: two dims
    uint4 c[4];
    uint32_t m[4][GSMAX];
};
template <int G> struct VRegs {
    static constexpr int MV = 2 * (kD / G);              // V meta words per lane of the largest unit (2 bits)
    uint4 c[4];
    uint32_t m[MV];
};

// Loads through a scalar base plus a 32-bit per-lane byte offset (no 64-bit vector address
// arithmetic: the base of every KiB is computed on the scalar unit).  The cache is read exactly once
// per call, so every load of it is a streaming (nontemporal) load: a plain read-only kernel moves
// 6.9 TB/s with them on this chip and 6.0 TB/s with ordinary loads.
__device__ __forceinline__ uint4 ld16(const uint8_t *sbase, uint32_t voff) {
    const v4u v = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(sbase + voff));
    return uint4{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ uint32_t ld4(const uint8_t *sbase, uint32_t voff) {
    return __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(sbase + voff));
}

// The V side: the 16-byte slots 64*j + l of the unit's V KiBs and its (token, group) meta
// words 64*jj + l, same conventions.
// SMALL (chunks of 8, 16 or 32 tokens, one unit per quantised chunk): the chunk is one token block of QD = 1, 2 or
// 4 slices, its V codes are 2 (8 bits: 4) tiles of 16*QD slots.  With QD < 4 lanes 0..16*QD-1 take tile i into c[i]
// as the lanes of the first slices of a full block would; the lanes of the absent slices and the registers of the
// absent tiles / second block hold zeros.  The meta words of a short chunk are fewer than 64: the lanes past
// them read the last one (their tokens have weight 0).
template <int G, bool SMALL>
__device__ __forceinline__ void load_v(const Unit &u, int lane, VRegs<G> &v, int N) {
    constexpr int NG = kD / G;
    const int nw = u.nvalid * NG;                                         // SMALL: meta words of the unit (u.nsub counts whole KiB of codes)
    const uint32_t vv = u.vc + (uint32_t)lane * 16u, vmo = u.vm + (uint32_t)(SMALL ? min(lane, nw - 1) : lane) * 4u;
    const int nvm = u.lgb == 4 ? 1 : (SMALL ? max(nw >> 6, 1) : (u.nsub * NG) >> u.lgb);   // rows of 64 meta words, >= 1
    // slots per tile (64 for whole 1-KiB tiles) and tiles of the chunk's one block; one code path for both shapes, so
    // that the waits on the loads around these can be counted exactly
    const int ts = SMALL && u.lgb < 4 ? min(64, (max(N, u.lgb == 1 ? 16 : 8) << 4) >> (u.lgb == 1 ? 4 : 3)) : 64;
    const bool part = SMALL && ts < 64;
    const int ntile = u.lgb == 3 ? 4 : 2;
    const uint32_t vh = u.vc + (uint32_t)(lane & (ts - 1)) * 16u;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const uint4 t = ld16(u.vb, vh + (part ? (uint32_t)(min(i, ntile - 1) * ts) * 16u : (uint32_t)min(i, u.nsub - 1) * 1024u));
        const bool ok = !part || (lane < ts && i < ntile);
        v.c[i] = SMALL ? uint4{ok ? t.x : 0u, ok ? t.y : 0u, ok ? t.z : 0u, ok ? t.w : 0u} : t;
    }
#pragma unroll
    for (int jj = 0; jj < VRegs<G>::MV; jj++) v.m[jj] = ld4(u.vb, vmo + (uint32_t)min(jj, nvm - 1) * 256u);
}

// Softmax weights of a quantised unit: fp16(p * V scale / pair scale) per (head, group, token) into LDS.
template <int BITS, int G, int REP, int NWV>
__device__ __forceinline__ void value_weights(const VRegs<G> &v, int lane, int wave,
                                              AttnLds<G, REP, NWV> &L, WaveState<REP> &st) {
    using B = BW<BITS>;
    constexpr int NG = kD / G;
    constexpr int MAXVM = (4 * B::TT * NG / 64) > 0 ? (4 * B::TT * NG / 64) : 1;
    // ---- softmax weights, one lane per V (token, group) meta word
    constexpr int n = 32 / BITS;
#pragma unroll
    for (int jj = 0; jj < MAXVM; jj++) {
        const int idx = 64 * jj + lane, tv = idx / NG, g = idx % NG;
        const float sV = half_bits_to_float(v.m[jj] & 0xffffu);
        const float zV = half_bits_to_float(v.m[jj] >> 16);
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
}

// ---- one unit of raw fp16 rows (16-bit chunks and the FP16 residual) -----------------------
// 16 rows: lane l holds dims 8*(l%16)..+7 of row 4*j + l/16, for K and for V alike.  Every lane of
// a row ends up with the row's score, so the weights need no trip through LDS: the score phase
// leaves p[r][j] in registers for the value phase.
// Several queries per sequence (nq > 1; head r belongs to query r / rep_in): query t does not see the residual rows of
// the queries after it, the last nq - 1 - t valid rows.
template <int G, int REP, int NWV, typename KR>
__device__ __forceinline__ void fp16_scores(const Unit &u, const KR &k, int lane, float scale_log2, int nq, int rep_in,
                                            AttnLds<G, REP, NWV> &L, WaveState<REP> &st, float (&p4)[REP][4]) {
    const int part = lane & 15, tok_l = lane >> 4;
#pragma unroll
    for (int r = 0; r < REP; r++) {
        const int nvalid = REP == 1 ? u.nvalid : min(u.nvalid, u.tail_rows - (nq - 1 - r / rep_in));   // an fp16 unit spans 16 rows
        const uint4 qv = *reinterpret_cast<const uint4 *>(&L.qtab[r][part * 4]);
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
        rescale<G, REP>(st, r, wave_max(lmax), lane);
#pragma unroll
        for (int j = 0; j < 4; j++) {
            p4[r][j] = (s4[j] == -INFINITY) ? 0.0f : fast_exp2(s4[j] - st.m[r]);   // masked rows
            if (part == 0) st.lsum[r] += p4[r][j];
        }
    }
}
template <int G, int REP, int NWV>
__device__ __forceinline__ void fp16_values(const Unit &u, const VRegs<G> &v, int lane, int wave,
                                            AttnLds<G, REP, NWV> &L, WaveState<REP> &st, const float (&p4)[REP][4]) {
    const int tok_l = lane >> 4;
    const int nvalid = u.nvalid;
    // staging buffer of the wavefront, 2 KiB: [row group l/16][half of the lane's 8 dims][column block l%16][4];
    // with four or more heads it lies over the weight rows, which only quantised units use
    float *stage;
    if constexpr (REP >= 4) stage = reinterpret_cast<float *>(&L.wl[wave][0][0][0]);
    else                    stage = &L.vf[wave][0];
    static_assert(REP < 4 || sizeof(L.wl[0]) >= 2048, "staging buffer");
#pragma unroll
    for (int r = 0; r < REP; r++) {
        float acc8[8];
#pragma unroll
        for (int e = 0; e < 8; e++) acc8[e] = 0.0f;
        // the packed halves feed the multiply-add directly (mixed-precision FMA), nothing is unpacked
        if (nvalid == 16) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float p24 = p4[r][j] * kTwoM24;                 // accumulators carry a factor 2^-24
                const uint32_t w[4] = {v.c[j].x, v.c[j].y, v.c[j].z, v.c[j].w};
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const half2_t h = as_half2(w[e >> 1]);
                    acc8[e] = fmaf(p24, (float)((e & 1) ? h.y : h.x), acc8[e]);
                }
            }
        } else {                                                      // the last rows of the residual
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float p24 = p4[r][j] * kTwoM24;
                const bool ok = 4 * j + tok_l < nvalid;               // rows past nvalid may hold NaN / Inf
                const uint32_t w[4] = {ok ? v.c[j].x : 0u, ok ? v.c[j].y : 0u, ok ? v.c[j].z : 0u, ok ? v.c[j].w : 0u};
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const half2_t h = as_half2(w[e >> 1]);
                    acc8[e] = fmaf(p24, (float)((e & 1) ? h.y : h.x), acc8[e]);
                }
            }
        }
        // fold the four row groups through LDS and hand every dim to the lane that owns it (2l, 2l+1)
        float4 t0, t1;
        t0.x = acc8[0]; t0.y = acc8[1]; t0.z = acc8[2]; t0.w = acc8[3];
        t1.x = acc8[4]; t1.y = acc8[5]; t1.z = acc8[6]; t1.w = acc8[7];
        float *mine_w = stage + (lane >> 4) * 128 + (lane & 15) * 4;
        *reinterpret_cast<float4 *>(mine_w) = t0;
        *reinterpret_cast<float4 *>(mine_w + 64) = t1;
        wave_sync();
        // dims 2l, 2l+1: column block l/4, element 2*(l%4) of its 8: half (l%4)/2, word 2*(l%2)
        const float *mine_r = stage + ((lane & 3) >> 1) * 64 + (lane >> 2) * 4 + (lane & 1) * 2;
        float2 s = *reinterpret_cast<const float2 *>(mine_r);
#pragma unroll
        for (int rg = 1; rg < 4; rg++) {
            const float2 t = *reinterpret_cast<const float2 *>(mine_r + rg * 128);
            s.x += t.x; s.y += t.y;
        }
        st.acc[r][0] += s.x;
        st.acc[r][1] += s.y;
        wave_sync();
    }
}

// ---- matrix-core path for grouped queries (REP > 1), quantised units -------------------------
// v_mfma_f32_16x16x32_f16 computes C[i][x] += sum_k A[i][k] B[k][x]; lane l = 16*qd + x holds
// A[x][8qd..8qd+7], B[8qd..8qd+7][x] and C[4qd..4qd+3][x].  Masked code words are valid B operands
// as they are (fp16 subnormals, which the matrix core keeps); the per-pair power of two and the
// 2^-24 are folded into A.  Tile rows carry (query head, group) pairs: row = head * NG + group.
//   scores: x = token of a 16-token tile, k = 32 dims (lane quarter qd holds dims 32qd + 8mi + 0..7 of
//           its token in pass mi = 0..3); A = q, zero outside the row's group.  The R = REP*NG rows in
//           use repeat 16/R times, so that many tiles are computed back to back and every lane keeps the
//           tile in which its own token lies: no lane is idle in the per-token arithmetic.
//   values: x = dim of a 16-dim column tile, k = 32 tokens (quarter qd holds its slice of the token
//           block); A = the softmax weights from LDS, rows >= R read zeros.
template <int G, int REP> struct MC {
    static constexpr int NG = kD / G;
    static constexpr int R = REP * NG;                   // tile rows in use
    static constexpr int F = 16 / (R < 16 ? R : 16);     // score tiles per pass
    static constexpr int HPL = 4 / NG;                   // query heads per lane (C register n: head n / NG)
    static constexpr int NSMAX = 8 / F;                  // passes of the largest unit (128 tokens, 8 tiles)
    __device__ static __forceinline__ int sel(int qd) { return F == 4 ? qd : (F == 2 ? (qd >> 1) : 0); }
    __device__ static __forceinline__ int slot0(int qd) { return (4 * qd) % R; }   // (head, group) slot of C register 0
};

template <int G, int REP> struct KRegsMC {
    uint4 c[4];
    uint32_t m[MC<G, REP>::NSMAX * (kD / G)];            // K meta words of the lane's own tokens
};

__device__ __forceinline__ v4f mfma16(v4u a, v4u b, v4f c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
}
__device__ __forceinline__ uint2 ld8(const uint8_t *sbase, uint32_t voff) {
    typedef uint32_t v2u __attribute__((ext_vector_type(2)));
    const v2u v = __builtin_nontemporal_load(reinterpret_cast<const v2u *>(sbase + voff));
    return uint2{v[0], v[1]};
}
// the k-th fp16 pair of a code word, left where it lies (scaled by 2^pair_exp(k))
template <int BITS> __device__ __forceinline__ uint32_t pair_reg(uint32_t w, int k) {
    using B = BW<BITS>;
    return k < B::KD ? (w & (B::MASK << (BITS * k))) : ((w >> B::SH) & (B::MASK << (BITS * (k - B::KD))));
}
template <int G, int REP>
__device__ __forceinline__ uint32_t kword(const KRegsMC<G, REP> &k, int i) {
    const uint4 &c = k.c[i >> 2];
    return (i & 3) == 0 ? c.x : ((i & 3) == 1 ? c.y : ((i & 3) == 2 ? c.z : c.w));
}
// pair index (inside its word) that feeds pair register pr of pass mi
template <int BITS> __device__ __forceinline__ constexpr int mc_pair(int mi, int pr) {
    return BITS == 2 ? 4 * (mi % 2) + pr : (BITS == 4 ? pr : pr % 2);
}
// B operand of score pass mi for token tile `tile`: the codes of dims 32qd + 8mi + 0..7
template <int BITS, int G, int REP>
__device__ __forceinline__ v4u mc_kcodes(const KRegsMC<G, REP> &k, int tile, int mi) {
    v4u b;
    if constexpr (BITS == 2) {
        const uint32_t w = kword(k, 2 * tile + mi / 2);
#pragma unroll
        for (int pr = 0; pr < 4; pr++) b[pr] = pair_reg<2>(w, mc_pair<2>(mi, pr));
    } else if constexpr (BITS == 4) {
        const uint32_t w = kword(k, 4 * tile + mi);
#pragma unroll
        for (int pr = 0; pr < 4; pr++) b[pr] = pair_reg<4>(w, pr);
    } else {
        const uint32_t w0 = kword(k, 8 * tile + 2 * mi), w1 = kword(k, 8 * tile + 2 * mi + 1);
        b[0] = pair_reg<8>(w0, 0); b[1] = pair_reg<8>(w0, 1); b[2] = pair_reg<8>(w1, 0); b[3] = pair_reg<8>(w1, 1);
    }
    return b;
}

// A operands of the score passes for the three quantised bit-widths, from the raw fp16 queries in LDS.
template <int G, int REP, typename LDS>
__device__ __forceinline__ void mc_build_q(const uint32_t *qraw32, int lane, int mi, LDS &L) {
    using M = MC<G, REP>;
    const int i = lane & 15, qd = lane >> 4;
    const int slot = i % M::R, r = slot / M::NG, g = slot % M::NG;
    const bool own = g == (32 * qd) / G;                 // the quarter's dims lie in the row's group
    {                                                    // pass mi: one wavefront per pass
        v4u ak[3];
#pragma unroll
        for (int pr = 0; pr < 4; pr++) {
            const uint32_t qq = qraw32[r * 64 + 16 * qd + 4 * mi + pr];          // dims 32qd + 8mi + 2pr, +1
            const float q0 = half_bits_to_float(qq & 0xffffu), q1 = half_bits_to_float(qq >> 16);
#pragma unroll
            for (int bi = 0; bi < 3; bi++) {
                const int kp = bi == 0 ? pair_exp<2>(mc_pair<2>(mi, pr)) : (bi == 1 ? pair_exp<4>(mc_pair<4>(mi, pr)) : 0);   // mi & 1 decides
                const float f = __builtin_bit_cast(float, (uint32_t)(127 - kp) << 23);
                const uint32_t v = float_to_half_bits(q0 * f) | (float_to_half_bits(q1 * f) << 16);
                ak[bi][pr] = own ? v : 0u;
            }
        }
#pragma unroll
        for (int bi = 0; bi < 3; bi++) L.qmc[bi][mi][lane] = ak[bi];
    }
}

// K side of a unit for grouped queries.  Quantised units: lane (x, qd) takes quarter qd of the code row
// of token 16*tile + x for every tile, and the meta words of its own tokens; raw fp16 units keep the
// slot order of load_k.  Eight 8-byte loads whatever the bit-width, branch-free like load_k.
template <int G, int REP, bool SMALL>
__device__ __forceinline__ void load_k_mc(const Unit &u, int lane, KRegsMC<G, REP> &k) {
    using M = MC<G, REP>;
    const int x = lane & 15, qd = lane >> 4;
    const bool raw = u.lgb == 4;
    const int rbsh = 4 + u.lgb;                           // log2(bytes of a code row)
    const uint32_t lane_off = raw ? (uint32_t)lane * 16u : (((uint32_t)x << rbsh) + ((uint32_t)qd << (rbsh - 2)));
    const int iptsh = raw ? 1 : u.lgb - 1;                // log2(loads per tile); raw: per KiB
    const int tbsh = raw ? 10 : rbsh + 4;                 // log2(bytes per tile); raw: a KiB
    // A streaming load drops its 128-byte line after use, so every line must be covered by ONE load instruction:
    // 8-byte pieces only at 2 bits (a quarter row is 8 bytes; the 16 lanes of a quarter cover whole lines together),
    // 16-byte pieces otherwise (a quarter row is 16 bytes at 4 bits, 32 bytes = two adjacent pieces at 8 bits).
    if (u.lgb == 1) {
        const int imax = 2 * u.nsub - 1;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int ic = min(i, imax);
            const uint2 t = ld8(u.kb, u.kc + lane_off + (((uint32_t)(ic >> iptsh) << tbsh) + (uint32_t)(ic & ((1 << iptsh) - 1)) * 8u));
            if (i & 1) { k.c[i >> 1].z = t.x; k.c[i >> 1].w = t.y; } else { k.c[i >> 1].x = t.x; k.c[i >> 1].y = t.y; }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            // 8 bits: a tile of 16 tokens is two pieces per lane, also when the chunk has only 8 tokens (1 KiB)
            const uint32_t jc = (uint32_t)min(j, (SMALL && u.lgb == 3 ? max(u.nsub, 2) : u.nsub) - 1);
            k.c[j] = ld16(u.kb, u.kc + lane_off + (u.lgb == 3 ? (jc >> 1) * 2048u + (jc & 1u) * 16u : jc * 1024u));
        }
    }
    const int TU = raw ? 16 : u.nvalid;                   // tokens of the unit
#pragma unroll
    for (int s = 0; s < M::NSMAX; s++) {
        const int t = min(16 * (s * M::F + M::sel(qd)) + x, TU - 1);
        if constexpr (M::NG == 2) {
            const uint2 mm = ld8(u.kb, u.km + (uint32_t)t * 8u);
            k.m[2 * s] = mm.x; k.m[2 * s + 1] = mm.y;
        } else {
            const uint4 mm = ld16(u.kb, u.km + (uint32_t)t * 16u);
            k.m[4 * s] = mm.x; k.m[4 * s + 1] = mm.y; k.m[4 * s + 2] = mm.z; k.m[4 * s + 3] = mm.w;
        }
    }
}

// Scores of a quantised unit -> L.sc (log2 domain), running maxima updated.
template <int BITS, int G, int REP, int NWV>
__device__ __forceinline__ void mc_scores(const Unit &u, const KRegsMC<G, REP> &k, const v4u (&ak)[4],
                                          const float (&qp)[4], int lane, int wave, float scale24,
                                          AttnLds<G, REP, NWV> &L, WaveState<REP> &st) {
    using M = MC<G, REP>;
    using B = BW<BITS>;
    constexpr int NG = M::NG, HPL = M::HPL, F = M::F;
    constexpr int TL = 16 / BITS;                         // tiles of a full unit: 8, 4, 2
    constexpr int NS = (TL + F - 1) / F;
    const int x = lane & 15, qd = lane >> 4, sel = M::sel(qd);
    const int TU = u.nvalid;
    float sv[NS][HPL], hmax[HPL];
#pragma unroll
    for (int h = 0; h < HPL; h++) hmax[h] = -INFINITY;
#pragma unroll
    for (int s = 0; s < NS; s++) {
        v4f own = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int f = 0; f < F; f++) {
            const int tile = s * F + f;
            if (tile < TL) {
                v4f c = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int mi = 0; mi < 4; mi++) c = mfma16(ak[mi], mc_kcodes<BITS, G, REP>(k, tile, mi), c);
                if (F == 1) own = c;
                else {
#pragma unroll
                    for (int n = 0; n < 4; n++) own[n] = (sel == f) ? c[n] : own[n];
                }
            }
        }
        const int t = 16 * (s * F + sel) + x;
        const bool valid = t < TU;
#pragma unroll
        for (int h = 0; h < HPL; h++) {
            float ps = 0.0f;
#pragma unroll
            for (int g = 0; g < NG; g++) {
                const uint32_t mw = k.m[s * NG + g];
                ps = fmaf(half_bits_to_float(mw & 0xffffu), own[h * NG + g], ps);
                ps = fmaf(half_bits_to_float(mw >> 16), qp[h * NG + g], ps);
            }
            sv[s][h] = valid ? ps * scale24 : -INFINITY;
            hmax[h] = fmaxf(hmax[h], sv[s][h]);
        }
    }
#pragma unroll
    for (int h = 0; h < HPL; h++) hmax[h] = group_max<16>(hmax[h]);
#pragma unroll
    for (int r = 0; r < REP; r++) {                       // the quarters whose rows hold head r
        float um = -INFINITY;
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
            const int r0q = ((4 * q4) % M::R) / NG;
            if (r0q <= r && r < r0q + HPL)
                um = fmaxf(um, __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, hmax[r - r0q]), 16 * q4)));
        }
        rescale<G, REP>(st, r, um, lane);
    }
    const int r0 = M::slot0(qd) / NG;
#pragma unroll
    for (int s = 0; s < NS; s++) {
        const int t = 16 * (s * F + sel) + x;
#pragma unroll
        for (int h = 0; h < HPL; h++) L.sc[wave][r0 + h][t] = sv[s][h];
    }
    wave_sync();
}

// Weighted value sum of a quantised unit on the matrix cores.
template <int BITS, int G, int REP, int NWV>
__device__ __forceinline__ void mc_value_dots(const VRegs<G> &v, int lane, int wave,
                                              AttnLds<G, REP, NWV> &L, WaveState<REP> &st) {
    using M = MC<G, REP>;
    constexpr int TW = 32 / BITS, TQ = TW > 8 ? TW : 8, WD = TQ / TW, CPK = 4 / WD, TB = 4 * TQ, KPB = 8 / CPK;
    constexpr int WLS = AttnLds<G, REP, NWV>::WLS;
    const int i = lane & 15, qd = lane >> 4;
    const uint16_t *arow = (i < M::R) ? &L.wl[wave][0][0][0] + i * WLS : &L.zrow[0];   // row = head * NG + group
    arow += qd * TQ;
    v4u a0 = {0, 0, 0, 0}, a1 = {0, 0, 0, 0};
#pragma unroll
    for (int jk = 0; jk < 4; jk++) {
        const int bu = jk / KPB, cg = jk % KPB;
        if (cg == 0) {                                    // the weights of this token block
            a0 = *reinterpret_cast<const v4u *>(arow + bu * TB);
            if constexpr (BITS == 2) a1 = *reinterpret_cast<const v4u *>(arow + bu * TB + 8);
        }
        const uint32_t wv[4] = {v.c[jk].x, v.c[jk].y, v.c[jk].z, v.c[jk].w};
        if constexpr (BITS == 8) {
#pragma unroll
            for (int nc = 0; nc < 2; nc++) {
                const int ct = cg * CPK + nc;
                v4u b;
                b[0] = pair_reg<8>(wv[2 * nc], 0); b[1] = pair_reg<8>(wv[2 * nc], 1);
                b[2] = pair_reg<8>(wv[2 * nc + 1], 0); b[3] = pair_reg<8>(wv[2 * nc + 1], 1);
                st.accA[ct] = mfma16(a0, b, st.accA[ct]);
            }
        } else {
#pragma unroll
            for (int nw = 0; nw < 4; nw++) {
                const int ct = cg * CPK + nw;
                v4u b;
#pragma unroll
                for (int pr = 0; pr < 4; pr++) b[pr] = pair_reg<BITS>(wv[nw], pr);
                st.accA[ct] = mfma16(a0, b, st.accA[ct]);
                if constexpr (BITS == 2) {
#pragma unroll
                    for (int pr = 0; pr < 4; pr++) b[pr] = pair_reg<2>(wv[nw], 4 + pr);
                    st.accA[ct] = mfma16(a1, b, st.accA[ct]);
                }
            }
        }
    }
    wave_sync();
}

// ---- integer matrix-core path (one query head per KV head), quantised units ------------------
// v_mfma_i32_16x16x64_i8 computes C[i][x] += sum_k A[i][k] B[k][x] on signed bytes; lane l = 16*xq + x
// holds A[x][16xq..16xq+15], B[16xq..16xq+15][x] and C[4xq..4xq+3][x].  The codes are the B operand:
// masking a code word byte-wise leaves one code per byte (2 bits: four planes, the code shifted left
// by 0, 2, 4, 5 bits; 4 bits: the low and the high nibbles; 8 bits: the bytes themselves, minus 128
// through a sign flip).  The other factor -- q for the scores, softmax weight * V scale for the values --
// is turned into a fixed-point integer, multiplied by the power of two that undoes its plane's shift,
// and split into four base-128 digits that sit in four rows of A; the four digit sums come back in the
// four C registers of a lane and are recombined exactly in integer / fp32 arithmetic.
//   scores: A is block diagonal (rows 4xq..4xq+3 are nonzero for k in quarter xq only), so that a lane's
//           C registers hold the dot product of its OWN 16 code bytes with the digits of q: the matrix
//           core serves as a per-lane 16-term integer dot product.  All lanes of a quarter must then hold
//           the same dims, which fixes the lane -> slot assignment of load_k_iq.
//   values: column x = dim of a 16-dim column tile, k = 64 tokens (quarter xq holds its slice of the token
//           block); rows 4g..4g+3 = digits of the weights of group g, so quarter g of the lanes ends up
//           with the sums for the column tiles whose dims lie in group g.
__device__ __forceinline__ v4i mfma_i8(v4i a, v4i b, v4i c) {
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}
// sum_n 128^n C[n] as fp32 (the two halves are exact integers below 2^31)
__device__ __forceinline__ float iq_combine(v4i c) {
    const int hi = c[3] * 128 + c[2], lo = c[1] * 128 + c[0];
    return fmaf((float)hi, 16384.0f, (float)lo);
}
// The byte planes of a code word.  2 bits: byte y of plane p holds code 8*(y%2) + 2p + y/2 of the word,
// shifted left by {0, 2, 4, 5}[p]; 4 bits: code 4*(y%2) + 2p + y/2; 8 bits: code 2*(y%2) + y/2, minus 128.
template <int BITS> struct IQ {
    static constexpr int NP = 8 / BITS;                  // planes of a word
    static constexpr int LGM = BITS == 2 ? 6 : 0;        // log2 of the factor every product carries
    static constexpr int BI = BITS == 2 ? 0 : (BITS == 4 ? 1 : 2);
    __device__ static __forceinline__ void planes(uint32_t w, int *m) {
        if constexpr (BITS == 2) {
            m[0] = (int)(w & 0x03030303u); m[1] = (int)(w & 0x0c0c0c0cu);
            m[2] = (int)(w & 0x30303030u); m[3] = (int)((w >> 1) & 0x60606060u);
        } else if constexpr (BITS == 4) {
            m[0] = (int)(w & 0x0f0f0f0fu); m[1] = (int)((w >> 4) & 0x0f0f0f0fu);
        } else {
            m[0] = (int)(w ^ 0x80808080u);
        }
    }
};
__device__ __forceinline__ uint32_t word_of(const uint4 &c, int i) {
    return i == 0 ? c.x : (i == 1 ? c.y : (i == 2 ? c.z : c.w));
}

// K side of a unit, one query head per KV head.  The codes are read in memory order (lane l takes the
// 16-byte slot 64j + l of KiB j, fully coalesced); iq_regroup then hands every lane the slot the matrix
// products want.  The meta words are read for the lane's final (token, group) directly:
//   2 bits: register j holds token 32j + 16*(xq/2) + c, half row xq%2 (64 dims);
//   4 bits: token 16j + c, quarter row xq (32 dims);
//   8 bits: token 16*(j/2) + c, eighth of a row 4*(j%2) + xq (16 dims);
// raw fp16 units keep the slot order and have no meta.
// KPC (keys quantised per channel): the meta words are [token group][dim]; lane l takes the words of dims 2l, 2l+1 of
// the (up to four) token groups the unit's tokens lie in.
template <int G, bool KPC, bool SMALL>
__device__ __forceinline__ void load_k_iq(const Unit &u, int lane, KRegs<G> &k) {
    constexpr int NG = kD / G;
    const uint32_t xq = (uint32_t)lane >> 4, c = (uint32_t)lane & 15u;
    const uint32_t vk = u.kc + (uint32_t)lane * 16u;
#pragma unroll
    for (int j = 0; j < 4; j++) k.c[j] = ld16(u.kb, vk + (uint32_t)min(j, u.nsub - 1) * 1024u);   // short unit: the last KiB is read again (ignored)
    if constexpr (KPC) {                                  // four loads for every unit (a raw fp16 unit reads its own rows and ignores them)
        const int lgq = min(u.lgb, 3);
        const int t0 = (int)(u.kc >> (4 + lgq)), TU = u.nsub << (6 - lgq);
        const int ngu = u.lgb == 4 ? 1 : (t0 % G + TU + G - 1) / G;
        const uint32_t mbase = u.lgb == 4 ? u.kc : u.km;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const uint2 mm = ld8(u.kb, mbase + (uint32_t)min(j, ngu - 1) * (kD * 4u) + (uint32_t)lane * 8u);
            k.m[j][0] = mm.x; k.m[j][1] = mm.y;
        }
        return;
    }
    // The same number of loads whatever the unit (a raw fp16 unit reads four words of its rows and ignores them) and
    // no branch: the waits on everything requested after these loads can then be counted exactly.
    // word of the lane's (token, group) per bit-width, and the step from register j to j + 1 (8 bits: two steps)
    const uint32_t w1 = (16u * (xq >> 1) + c) * NG + (xq & 1u) * (NG / 2);
    const uint32_t w2 = c * NG + (NG == 2 ? (xq >> 1) : xq);
    const uint32_t w3 = c * NG + (NG == 2 ? 0u : (xq >> 1));
    const uint32_t vm = u.lgb == 4 ? u.kc + c * 4u : u.km + (u.lgb == 1 ? w1 : (u.lgb == 2 ? w2 : w3)) * 4u;
    const int jmax = (SMALL || u.lgb == 1) ? u.nsub - 1 : 3;   // a short unit's block ends early
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const uint32_t jc = (uint32_t)min(j, jmax);
        const uint32_t o1 = jc * (32u * NG * 4u), o2 = jc * (16u * NG * 4u);
        const uint32_t o3 = (uint32_t)(j >> 1) * (16u * NG * 4u) + (uint32_t)(j & 1) * ((NG / 2) * 4u);
        const uint32_t oj = u.lgb == 4 ? 0u : (u.lgb == 1 ? o1 : (u.lgb == 2 ? o2 : o3));
        k.m[j][0] = ld4(u.kb, vm + oj);
        if constexpr (NG == 4) k.m[j][1] = ld4(u.kb, vm + oj + (u.lgb == 1 ? 4u : 0u));
    }
}

// Hands every lane the code slots of its (token, part) through the wavefront's LDS buffer.  The slots
// are stored XOR-swizzled (and every KiB 128 bytes further than the last), so that both the writes in
// memory order and the regrouped reads touch every bank once.
template <int BITS, int G, int NWV>
__device__ __forceinline__ void iq_regroup(const KRegs<G> &k, int lane, int wave, AttnLds<G, 1, NWV> &L, uint4 (&kc)[4]) {
    constexpr int KS = 72;                                // slots between two KiBs
    uint4 *buf = &L.kx[wave][0];
    const int xq = lane >> 4, c = lane & 15;
    const int sw = BITS == 2 ? (lane >> 4) & 1 : (BITS == 4 ? (lane >> 4) & 3 : (lane >> 3) & 7);
#pragma unroll
    for (int j = 0; j < 4; j++) buf[j * KS + (lane ^ sw)] = k.c[j];
    wave_sync();
#pragma unroll
    for (int j = 0; j < 4; j++) {
        int pos;
        if constexpr (BITS == 2)      pos = j * KS + ((32 * (xq >> 1) + 2 * c + (xq & 1)) ^ (c >> 3));
        else if constexpr (BITS == 4) pos = j * KS + 4 * c + (xq ^ (c >> 2));
        else                          pos = (2 * (j >> 1) + (c >> 3)) * KS + 8 * (c & 7) + ((4 * (j & 1) + xq) ^ (c & 7));
        kc[j] = buf[pos];
    }
    wave_sync();
}

// Scores of a quantised unit -> L.sc (log2 domain), running maximum updated.
// SMALL: the unit may hold fewer tokens than a KiB of codes does (chunks of 8 and 16 tokens); the scores of the
// tokens past u.nvalid are masked one by one.
template <int BITS, int G, int NWV, bool SMALL>
__device__ __forceinline__ void iq_scores(const Unit &u, const KRegs<G> &k, int lane, int wave,
                                          AttnLds<G, 1, NWV> &L, WaveState<1> &st) {
    constexpr int NG = kD / G;
    const int xq = lane >> 4, c = lane & 15;
    const float sc = L.iqscale[IQ<BITS>::BI];
    const v4i zero = {0, 0, 0, 0};
    uint4 kc[4];
    iq_regroup<BITS, G, NWV>(k, lane, wave, L, kc);
    if constexpr (BITS == 2) {
        constexpr int GS = NG == 4 ? 2 : 1;              // groups inside a half row
        const int part = xq & 1;
        v4i A[4];
#pragma unroll
        for (int wd = 0; wd < 4; wd++) A[wd] = L.qa[wd][lane];
        float qp[GS];
#pragma unroll
        for (int gi = 0; gi < GS; gi++) qp[gi] = L.iqpart[0][part][gi];
        float s4[4], lmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            v4i acc[GS];
#pragma unroll
            for (int gi = 0; gi < GS; gi++) acc[gi] = zero;
#pragma unroll
            for (int wd = 0; wd < 4; wd++) {
                int m[4];
                IQ<2>::planes(word_of(kc[j], wd), m);
                acc[wd / (4 / GS)] = mfma_i8(A[wd], v4i{m[0], m[1], m[2], m[3]}, acc[wd / (4 / GS)]);
            }
            float ps = 0.0f;
#pragma unroll
            for (int gi = 0; gi < GS; gi++) {
                ps = fmaf(half_bits_to_float(k.m[j][gi] & 0xffffu), iq_combine(acc[gi]), ps);
                ps = fmaf(half_bits_to_float(k.m[j][gi] >> 16), qp[gi], ps);
            }
            ps += __shfl_xor(ps, 16);
            const bool ok = SMALL ? 32 * j + 16 * (xq >> 1) + c < u.nvalid : j < u.nsub;   // KiB past a short unit: ignored
            s4[j] = ok ? ps * sc : -INFINITY;
            lmax = fmaxf(lmax, s4[j]);
        }
        rescale<G, 1>(st, 0, wave_max(lmax), lane);
        if (part == 0) {
#pragma unroll
            for (int j = 0; j < 4; j++) L.sc[wave][0][32 * j + 16 * (xq >> 1) + c] = s4[j];
        }
    } else if constexpr (BITS == 4) {
        const v4i A0 = L.qa[4][lane], A1 = L.qa[5][lane];
        const float qp = L.iqpart[1][xq][0];
        float s4[4], lmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            int m0[2], m1[2], m2[2], m3[2];
            IQ<4>::planes(kc[j].x, m0); IQ<4>::planes(kc[j].y, m1);
            IQ<4>::planes(kc[j].z, m2); IQ<4>::planes(kc[j].w, m3);
            v4i acc = mfma_i8(A0, v4i{m0[0], m0[1], m1[0], m1[1]}, zero);
            acc = mfma_i8(A1, v4i{m2[0], m2[1], m3[0], m3[1]}, acc);
            float ps = half_bits_to_float(k.m[j][0] >> 16) * qp;
            ps = fmaf(half_bits_to_float(k.m[j][0] & 0xffffu), iq_combine(acc), ps);
            ps += __shfl_xor(ps, 16);
            ps += __shfl_xor(ps, 32);
            const bool ok = SMALL ? 16 * j + c < u.nvalid : j < u.nsub;   // KiB past a short unit: ignored
            s4[j] = ok ? ps * sc : -INFINITY;
            lmax = fmaxf(lmax, s4[j]);
        }
        rescale<G, 1>(st, 0, wave_max(lmax), lane);
        if (xq == 0) {
#pragma unroll
            for (int j = 0; j < 4; j++) L.sc[wave][0][16 * j + c] = s4[j];
        }
    } else {
        const v4i A[2] = {L.qa[6][lane], L.qa[7][lane]};
        const float qp[2] = {L.iqpart[2][xq][0], L.iqpart[2][4 + xq][0]};
        float s2[2], lmax = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < 2; jj++) {
            float ps = 0.0f;
#pragma unroll
            for (int r = 0; r < 2; r++) {
                const uint4 &w = kc[2 * jj + r];
                const v4i b = {(int)(w.x ^ 0x80808080u), (int)(w.y ^ 0x80808080u), (int)(w.z ^ 0x80808080u), (int)(w.w ^ 0x80808080u)};
                const float isum = fmaf(128.0f, qp[r], iq_combine(mfma_i8(A[r], b, zero)));
                const uint32_t mw = k.m[2 * jj + r][0];
                ps = fmaf(half_bits_to_float(mw & 0xffffu), isum, ps);
                ps = fmaf(half_bits_to_float(mw >> 16), qp[r], ps);
            }
            ps += __shfl_xor(ps, 16);
            ps += __shfl_xor(ps, 32);
            s2[jj] = (!SMALL || 16 * jj + c < u.nvalid) ? ps * sc : -INFINITY;
            lmax = fmaxf(lmax, s2[jj]);
        }
        rescale<G, 1>(st, 0, wave_max(lmax), lane);
        if (xq == 0) { L.sc[wave][0][c] = s2[0]; L.sc[wave][0][16 + c] = s2[1]; }
    }
    wave_sync();
}

// Scores of a quantised unit whose keys are quantised per channel (a group = G consecutive tokens of one dim):
//   q . k^_t = sum_d (q_d * scale_{g,d}) * code_{t,d} + sum_d q_d * zero_{g,d},   g = the token group of t,
// so the scale folds into a copy of q per token group (built here from the unit's meta words and kept in LDS)
// and the zero-points into one number per group.  The codes stay in the slots as loaded (lane l holds slot 64j + l
// of KiB j = part l % SPR of a token's row); the dot products run on the vector ALU, one multiply-add per code,
// and the SPR lanes of a token are summed by DPP.  Result as iq_scores: L.sc (log2 domain), running maximum updated.
template <int BITS, int G, int NWV>
__device__ __forceinline__ void pc_scores(const Unit &u, const KRegs<G> &k, int lane, int wave, float scale_log2,
                                          AttnLds<G, 1, NWV> &L, WaveState<1> &st) {
    constexpr int E = 128 / BITS, SPR = BITS, CPW = 32 / BITS;
    constexpr int NGU = (256 / BITS) / G > 0 ? (256 / BITS) / G : 1;     // token groups a full unit spans
    const uint32_t qq = L.qraw[lane];
    const float q0 = half_bits_to_float(qq & 0xffffu), q1 = half_bits_to_float(qq >> 16);
    float bias[NGU];
#pragma unroll
    for (int j = 0; j < NGU; j++) {
        const uint32_t m0 = k.m[j][0], m1 = k.m[j][1];
        float2 qs;
        qs.x = q0 * half_bits_to_float(m0 & 0xffffu); qs.y = q1 * half_bits_to_float(m1 & 0xffffu);
        *reinterpret_cast<float2 *>(&L.pcq[wave][j][2 * lane]) = qs;
        float bz = fmaf(q0, half_bits_to_float(m0 >> 16), q1 * half_bits_to_float(m1 >> 16));
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) bz += __shfl_xor(bz, o);
        bias[j] = bz;
    }
    wave_sync();
    const int part = lane % SPR;
    const int goff = (int)(u.kc >> (4 + u.lgb)) % G;      // tokens of the unit's first token group that lie before the unit
    float s4[4], lmax = -INFINITY;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const int tk = (64 * j + lane) / SPR;             // token of the slot, counted inside the unit
        const int gj = NGU > 1 ? (goff + tk) / G : 0;
        const float *qp = &L.pcq[wave][gj][E * part];
        float dot = 0.0f;
#pragma unroll
        for (int wd = 0; wd < 4; wd++) {
            const uint32_t w = word_of(k.c[j], wd);
#pragma unroll
            for (int e4 = 0; e4 < CPW / 4; e4++) {
                const float4 qv = *reinterpret_cast<const float4 *>(qp + wd * CPW + 4 * e4);
                const float qa[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const int e = 4 * e4 + i;
                    const uint32_t code = (w >> (16 * (e & 1) + BITS * (e >> 1))) & ((1u << BITS) - 1u);
                    dot = fmaf((float)code, qa[i], dot);
                }
            }
        }
        dot = group_sum<SPR>(dot);
        float bz = bias[0];
#pragma unroll
        for (int g = 1; g < NGU; g++) bz = (gj == g) ? bias[g] : bz;
        s4[j] = (j < u.nsub) ? (dot + bz) * scale_log2 : -INFINITY;      // KiB past a short unit: ignored
        lmax = fmaxf(lmax, s4[j]);
    }
    rescale<G, 1>(st, 0, wave_max(lmax), lane);
    if (part == 0) {
#pragma unroll
        for (int j = 0; j < 4; j++) L.sc[wave][0][(64 * j + lane) / SPR] = s4[j];
    }
    wave_sync();
}

// Softmax weights of a quantised unit as the A operand of the value products: one lane per V (token,
// group) meta word computes p * V scale, the wavefront agrees on a common power of two, and the four
// base-128 digits of the fixed-point weight go to the rows 4g..4g+3 of the operand image in LDS.
// Returns the factor that turns the recombined digit sums back into weights * codes.
template <int BITS, int G, int NWV>
__device__ __forceinline__ float iq_weights(const VRegs<G> &v, int lane, int wave,
                                            AttnLds<G, 1, NWV> &L, WaveState<1> &st) {
    constexpr int NG = kD / G;
    constexpr int MV = (256 / BITS) * NG / 64;           // meta words per lane: tokens of a unit * groups / 64
    float wv[MV], wmax = 0.0f;
#pragma unroll
    for (int jj = 0; jj < MV; jj++) {
        const int idx = 64 * jj + lane, tv = idx / NG, g = idx % NG;
        const float sV = half_bits_to_float(v.m[jj] & 0xffffu);
        const float zV = half_bits_to_float(v.m[jj] >> 16);
        const float p = fast_exp2(L.sc[wave][0][tv] - st.m[0]);       // tokens past a short unit: score -inf, p = 0
        if (g == 0) st.lsum[0] += p;
        st.z[0] = fmaf(p, BITS == 8 ? fmaf(128.0f, sV, zV) : zV, st.z[0]);   // 8 bits: the codes enter minus 128
        wv[jj] = p * sV;
        wmax = fmaxf(wmax, wv[jj]);
    }
    wmax = wave_max(wmax);
    // 2^ef <= wmax < 2^(ef+1) (ef >= -100): weight * 2^(20 - ef) < 2^21
    const int ef = max((int)((__builtin_bit_cast(uint32_t, wmax) >> 23) & 255u) - 127, -100);
    const float up = __builtin_bit_cast(float, (uint32_t)(127 + 20 - ef) << 23);
    uint8_t *img = reinterpret_cast<uint8_t *>(&L.wa[wave][0][0]);
#pragma unroll
    for (int jj = 0; jj < MV; jj++) {
        const uint32_t pos = L.wpos[IQ<BITS>::BI][jj][lane];         // byte offset of digit 0 | plane shift << 16
        const uint32_t W = (uint32_t)(wv[jj] * up + 0.5f) << (pos >> 16);
        uint8_t *dst = img + (pos & 0xffffu);
        dst[0] = (uint8_t)(W & 127u); dst[16] = (uint8_t)((W >> 7) & 127u);
        dst[32] = (uint8_t)((W >> 14) & 127u); dst[48] = (uint8_t)((W >> 21) & 127u);
    }
    wave_sync();
    return __builtin_bit_cast(float, (uint32_t)(127 + ef - 20 - IQ<BITS>::LGM) << 23);
}

// Weighted value sum of a quantised unit on the integer matrix cores.
template <int BITS, int G, int NWV>
__device__ __forceinline__ void iq_values(const VRegs<G> &v, int lane, int wave, float cw,
                                          AttnLds<G, 1, NWV> &L, WaveState<1> &st) {
    const v4i zero = {0, 0, 0, 0};
    const v4i A0 = L.wa[wave][0][lane];
    if constexpr (BITS == 2) {                           // two blocks of 64 tokens; KiB j: block j/2, column tiles 4*(j%2)..+3
        const v4i A1 = L.wa[wave][1][lane];
#pragma unroll
        for (int ct = 0; ct < 8; ct++) {
            int m[4];
            IQ<2>::planes(word_of(v.c[ct / 4], ct % 4), m);
            v4i acc = mfma_i8(A0, v4i{m[0], m[1], m[2], m[3]}, zero);
            IQ<2>::planes(word_of(v.c[2 + ct / 4], ct % 4), m);
            acc = mfma_i8(A1, v4i{m[0], m[1], m[2], m[3]}, acc);
            st.accq[0][ct] = fmaf(iq_combine(acc), cw, st.accq[0][ct]);
        }
    } else if constexpr (BITS == 4) {                    // two blocks of 32 tokens share one product
#pragma unroll
        for (int ct = 0; ct < 8; ct++) {
            int ma[2], mb[2];
            IQ<4>::planes(word_of(v.c[ct / 4], ct % 4), ma);
            IQ<4>::planes(word_of(v.c[2 + ct / 4], ct % 4), mb);
            const v4i acc = mfma_i8(A0, v4i{ma[0], ma[1], mb[0], mb[1]}, zero);
            st.accq[0][ct] = fmaf(iq_combine(acc), cw, st.accq[0][ct]);
        }
    } else {                                             // one block of 32 tokens: half of the k range is unused
#pragma unroll
        for (int ct = 0; ct < 8; ct++) {
            const uint32_t w0 = word_of(v.c[ct / 2], 2 * (ct % 2)), w1 = word_of(v.c[ct / 2], 2 * (ct % 2) + 1);
            const v4i acc = mfma_i8(A0, v4i{(int)(w0 ^ 0x80808080u), (int)(w1 ^ 0x80808080u), 0, 0}, zero);
            st.accq[0][ct] = fmaf(iq_combine(acc), cw, st.accq[0][ct]);
        }
    }
    wave_sync();
}

// Tables of the integer path for the queries of one row (REP == 1), built by the whole workgroup
// once L.qraw is in place:  iq[d] = q_d as a fixed-point integer below 2^21 in magnitude, qa = the
// eight A operands of the score products (2 bits: word 0..3 of a slot; 4 bits: word pair 0, 1;
// 8 bits: register parity 0, 1), iqpart = sum of iq over a lane's dims inside one group (times the
// common factor of the bit-width), iqscale = softmax scale (log2 domain) / fixed-point factors.
template <int G, int NWV>
__device__ __forceinline__ void iq_build_q(AttnLds<G, 1, NWV> &L, int tid, int lane, float scale_log2) {
    constexpr int NT = NWV * 64;
    const uint32_t pr = L.qraw[lane];
    float qm = fmaxf(fabsf(half_bits_to_float(pr & 0xffffu)), fabsf(half_bits_to_float(pr >> 16)));
    qm = wave_max(qm);
    const int ef = qm > 0.0f ? (int)((__builtin_bit_cast(uint32_t, qm) >> 23) & 255u) - 127 : 0;   // 2^ef <= max |q| < 2^(ef+1)
    const float up = __builtin_bit_cast(float, (uint32_t)(127 + 20 - ef) << 23);
    const uint16_t *qraw = reinterpret_cast<const uint16_t *>(L.qraw);
    if (tid < 3) L.iqscale[tid] = scale_log2 * __builtin_bit_cast(float, (uint32_t)(127 + ef - 20 - (tid == 0 ? 6 : 0)) << 23);
    int s16 = 0;                                          // sums of iq over blocks of 16 dims (wavefronts 0 and 1)
    if (tid < kD) {
        s16 = L.iq[tid] = (int)rintf(half_bits_to_float(qraw[tid]) * up);
        s16 += (int)dpp_u<DPP_XOR1>((uint32_t)s16); s16 += (int)dpp_u<DPP_XOR2>((uint32_t)s16);
        s16 += (int)dpp_u<DPP_HALF_MIRROR>((uint32_t)s16); s16 += (int)dpp_u<DPP_MIRROR>((uint32_t)s16);
        if ((tid & 15) == 0) L.iqs16[tid >> 4] = s16;
    }
    __syncthreads();
    // the 16 lanes 20*xq + n of every operand are nonzero (the rest was zeroed once): one word per thread
    static_assert(NT == 512, "one operand word per thread");
    {
        const int t = tid >> 6, xq = (tid >> 4) & 3, n = (tid >> 2) & 3, m = tid & 3;
        uint32_t wd = 0u;
#pragma unroll
        for (int y = 0; y < 4; y++) {
            int d, sh = 0;                                // dim of byte 4m + y, power of two that undoes the plane's shift
            if (t < 4)      { d = (xq & 1) * 64 + t * 16 + 8 * (y & 1) + 2 * m + (y >> 1); sh = m == 3 ? 1 : 6 - 2 * m; }
            else if (t < 6) { d = xq * 32 + (2 * (t - 4) + (m >> 1)) * 8 + 4 * (y & 1) + 2 * (m & 1) + (y >> 1); }
            else            { d = (4 * (t - 6) + xq) * 16 + m * 4 + 2 * (y & 1) + (y >> 1); }
            const int Q = L.iq[d];
            const uint32_t mag = (uint32_t)(Q < 0 ? -Q : Q) << sh;
            int dg = (int)((mag >> (7 * n)) & 127u);
            if (Q < 0) dg = -dg;
            wd |= ((uint32_t)dg & 255u) << (8 * y);
        }
        reinterpret_cast<uint32_t *>(&L.qa[t][20 * xq + n])[m] = wd;
    }
    if (tid < 3 * 8 * 2) {
        const int bi = tid / 16, part = (tid / 2) % 8, gi = tid % 2;
        const int E = 64 >> bi;                           // codes of a slot
        const int gs = E > G ? E / G : 1;
        int sq = 0;
        if (part < (2 << bi) && gi < gs) {
            const int nb = E / gs / 16, b0 = (part * E + gi * (E / gs)) / 16;
            for (int k = 0; k < nb; k++) sq += L.iqs16[b0 + k];
        }
        L.iqpart[bi][part][gi] = (float)sq * (bi == 0 ? 64.0f : 1.0f);
    }
}

// Positions of the weight digits in the operand image, per bit-width and (meta word, lane): byte
// offset of digit 0 (digit n follows 16n bytes later) | shift that undoes the plane's << 16.
template <int G, int NWV>
__device__ __forceinline__ void iq_build_wpos(AttnLds<G, 1, NWV> &L, int tid) {
    constexpr int NT = NWV * 64, NG = kD / G;
    for (int i = tid; i < 3 * 8 * 64; i += NT) {
        const int bi = i / 512, jj = (i / 64) % 8, l = i % 64;
        const int idx = 64 * jj + l, tv = idx / NG, g = idx % NG;
        uint32_t pos = 0;
        if (tv < (128 >> bi)) {
            int blk = 0, xq, b, sh = 0;
            if (bi == 0)      { blk = tv >> 6; const int tb = tv & 63, e = tb & 15, p = (e & 7) >> 1;
                                xq = tb >> 4; b = 4 * p + (e >> 3) + 2 * (e & 1); sh = p == 3 ? 1 : 6 - 2 * p; }
            else if (bi == 1) { const int tb = tv & 31, e = tb & 7, p = (e & 3) >> 1;
                                xq = tb >> 3; b = 8 * (tv >> 5) + 4 * p + (e >> 2) + 2 * (e & 1); }
            else              { const int e = tv & 3;
                                xq = tv >> 3; b = 4 * ((tv & 7) >> 2) + (e >> 1) + 2 * (e & 1); }
            pos = (uint32_t)(blk * 1024 + (16 * xq + 4 * g) * 16 + b) | ((uint32_t)sh << 16);
        }
        L.wpos[bi][jj][l] = pos;
    }
    // operand lanes / rows of the image that nobody writes stay zero
    for (int i = tid; i < 8 * 64; i += NT) L.qa[i / 64][i % 64] = v4i{0, 0, 0, 0};
    for (int i = tid; i < NWV * 2 * 64; i += NT) L.wa[i / 128][(i / 64) % 2][i % 64] = v4i{0, 0, 0, 0};
}

// ---- work distribution ----------------------------------------------------------------------
// One persistent workgroup per CU slot.  The rows are laid end to end on an axis measured in bytes to
// read (row u covers [U[u], U[u+1]): the cost of its units, added up by attn_prep_kernel from the routing
// decisions), and workgroup w of NW owns the interval [w*Utot/NW, (w+1)*Utot/NW): part of a row, or
// several rows, always the same amount of work whatever the rows' mixes of bit-widths.  With more than
// kMaxWeightedRows rows every row counts the same (U[u] = u * NW) and many rows average out.
// Inside a row segment the workgroup's wavefronts draw tickets (one unit each) from counters shared by
// the workgroups of the row: a wavefront or workgroup that runs faster just takes more tickets, and
// all of them finish the row together.  The workgroup then folds its wavefronts' softmax states into
// ONE partial per row; partial slot of workgroup w in row u = w - (first workgroup that touches u).
constexpr int kMaxWeightedRows = 1024;
// Workgroups whose intervals meet row [ub, ue) (ue > ub): lo_w = floor(w*Utot/NW) < ue and lo_{w+1} > ub.
__device__ inline int wg_first_of_row(unsigned long long ub, unsigned long long Utot, int NW) {
    return (int)(((ub + 1) * (unsigned long long)NW + Utot - 1) / Utot) - 1;
}
__device__ inline int wg_last_of_row(unsigned long long ue, unsigned long long Utot, int NW) {
    return (int)((ue * (unsigned long long)NW + Utot - 1) / Utot) - 1;
}
// Partial slots per row.  A row's units are at most 8 times another's (16 against 2 bits), so a row
// holds at most 8/(BH+7) of all units and meets at most NW times that, plus two, intervals.
int attn_max_partials(int NW, int BH) {
    const int p = BH <= kMaxWeightedRows ? (8 * NW) / (BH + 7) + 3 : NW / BH + 2;
    return p < NW ? p : NW;
}
__device__ __forceinline__ int bits_of_expert(const AttnArgs &a, int e) {
    int b = 0;
#pragma unroll
    for (int k = 0; k < 8; k++) b = (e == k) ? a.bits_of[k] : b;
    return b;
}
__device__ __forceinline__ int lgb_of_bits(int bits) { return bits == 2 ? 1 : (bits == 4 ? 2 : (bits == 8 ? 3 : 4)); }
__device__ __forceinline__ uint32_t units_of_chunk(int N, int lgb) { return (uint32_t)((N + (256 >> lgb) - 1) >> (8 - lgb)); }

// Chunks per row segment: at most kDescCap, and at most kUnitCap units if all of them were FP16.
__host__ __device__ inline int attn_segment_chunks(int N) { return min(kDescCap, kUnitCap / max(N / 16, 1)); }

// RAGGED: the sequences of the batch have their own numbers of chunks and residual rows (a.seq_chunks,
// a.seq_tail, device arrays indexed by sequence); a.n_chunks is then the bound that sizes the segments.
// SMALL: chunks of 8, 16 or 32 tokens (a.N < 64), see load_v.  KPC: keys quantised per channel (REP == 1 only), see pc_scores.
template <int G, int REP, int NWV, bool RAGGED, bool SMALL, bool KPC>
__global__ __launch_bounds__(NWV * 64) void attn_split_kernel(AttnArgs a) {
    static_assert(!KPC || REP == 1, "per-channel keys: one query head per KV head");
    __shared__ AttnLds<G, REP, NWV> L;
    constexpr int NG = kD / G;
    constexpr int NT = NWV * 64;
    using KR = std::conditional_t<REP == 1, KRegs<G>, KRegsMC<G, REP>>;
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);           // wave-uniform, kept scalar
    const int w = (int)blockIdx.x, NW = (int)gridDim.x;
    const int N = a.N;

    auto bits_of = [&](int e) { return bits_of_expert(a, e); };

    const int seg_chunks = attn_segment_chunks(N);
    const int n_seg = max(1, (a.n_chunks + seg_chunks - 1) / seg_chunks);
    // ---- the workgroup's interval of the unit axis
    const bool weighted = a.BH <= kMaxWeightedRows;
    if (weighted) {                                      // U = inclusive scan of the rows' unit counts, two rows per thread
        static_assert(kMaxWeightedRows <= 2 * NT, "two rows per thread");
        const uint32_t *row_units = a.counters + (size_t)a.BH * n_seg * kCounterStride;
        const int i0 = 2 * tid;
        const uint32_t v0 = i0 < a.BH ? row_units[i0] : 0u, v1 = i0 + 1 < a.BH ? row_units[i0 + 1] : 0u;
        if constexpr (REP == 1) iq_build_wpos<G, NWV>(L, tid);          // behind the load
        const uint32_t incl = wave_incl_scan(v0 + v1);
        if (lane == 63) L.wscan[wave] = incl;
        __syncthreads();
        uint32_t excl = incl - (v0 + v1);
#pragma unroll
        for (int wv = 0; wv < NWV; wv++) if (wv < wave) excl += L.wscan[wv];
        if (tid == 0) { L.U[0] = 0u; L.r0 = 0u; }
        if (i0 < a.BH) L.U[i0 + 1] = excl + v0;
        if (i0 + 1 < a.BH) L.U[i0 + 2] = excl + v0 + v1;
        __syncthreads();
    } else {
        if constexpr (REP == 1) iq_build_wpos<G, NWV>(L, tid);          // made visible by the barriers of the row set-up
    }
    auto Uof = [&](int u) -> unsigned long long { return weighted ? (unsigned long long)L.U[u] : (unsigned long long)u * NW; };
    const unsigned long long Utot = Uof(a.BH);
    const unsigned long long lo = (unsigned long long)w * Utot / NW, hi = (unsigned long long)(w + 1) * Utot / NW;
    int r0 = (int)(lo / (unsigned long long)NW);         // the row that holds unit lo
    if (weighted) {
        for (int i = tid; i < a.BH; i += NT)
            if ((unsigned long long)L.U[i] <= lo && lo < (unsigned long long)L.U[i + 1]) L.r0 = (uint32_t)i;
        __syncthreads();
        r0 = (int)L.r0;
    }
    uint32_t *row_wgs = a.counters + (size_t)a.BH * n_seg * kCounterStride + a.BH;   // for the merge: workgroups per row
    for (int u = r0; u < a.BH && lo < hi && Uof(u) < hi; u++) {
        const unsigned long long ub = Uof(u), ue = Uof(u + 1), ru = ue - ub;
        if (ru == 0) continue;
        const uint8_t *erow = a.expert + (int64_t)u * a.desc_stride;
        const uint64_t *orow = a.chunk_off + (int64_t)u * a.desc_stride;
        int C = a.n_chunks, n_tail = a.n_tail;           // of this row
        if constexpr (RAGGED) {
            C = min(max(a.seq_chunks[u / a.Hkv], 0), a.n_chunks);
            n_tail = min(max(a.seq_tail[u / a.Hkv], 0), N - 1);
        }
        // workgroups that share this row's tickets, and the share of the row inside this workgroup's
        // interval: a workgroup whose interval covers only part of the row takes at most that part of
        // the tickets (it owes the rest of its time to the neighbouring row)
        const int wg_first = wg_first_of_row(ub, Utot, NW);
        const uint32_t P = (uint32_t)(wg_last_of_row(ue, Utot, NW) - wg_first + 1);
        const unsigned long long ov = min(hi, ue) - max(lo, ub);
        const bool whole = (lo >= ub && hi <= ue) || (ub >= lo && ue <= hi);   // the interval inside the row, or the row inside it
        if (w == wg_first && tid == 0) row_wgs[u] = P;

        // ---- (a) row set-up.  One round trip to memory for everything the first units need: the raw
        //      queries, the chunk descriptors of the first segment and the first batch of tickets.  The
        //      tables derived from q are built later, while the first units' codes are on their way.
        const int KPT = (seg_chunks + NT - 1) / NT;      // chunks per thread of a segment (<= 2)
        uint32_t q_first = 0u, g_first = 0u;
        uint8_t e_first[2] = {0, 0};
        uint64_t o_first[2] = {0ull, 0ull};
        {
            static_assert(REP * 64 <= NT, "one query word per thread");
            // head r of the row = query r / rep_in, query head (u % Hkv) * rep_in + r % rep_in of q [B, nq, Hkv * rep_in, D]
            if (tid < REP * 64) {
                const int r = tid >> 6, bq = u / a.Hkv;
                const int64_t qrow = ((int64_t)bq * a.nq + r / a.rep_in) * (a.Hkv * a.rep_in) + (u % a.Hkv) * a.rep_in + r % a.rep_in;
                q_first = reinterpret_cast<const uint32_t *>(a.q)[qrow * 64 + (tid & 63)];
            }
#pragma unroll
            for (int k = 0; k < 2; k++) {
                const int c = tid * KPT + k;
                if (k < KPT && c < min(C, seg_chunks)) { e_first[k] = erow[c]; o_first[k] = orow[c]; }
            }
            if (tid == 0) g_first = atomicAdd(a.counters + (size_t)u * n_seg * kCounterStride, (unsigned int)NWV);
            __syncthreads();                             // LDS of the previous row is free
            if (tid < REP * 64) L.qraw[tid] = q_first;
        }
        constexpr bool kLateTables = REP == 1;           // grouped queries: the builders would not fit beside the loads in flight
        auto build_q_tables = [&]() {                    // by the whole workgroup; L.qraw is in place
            const uint16_t *qraw = reinterpret_cast<const uint16_t *>(L.qraw);
            if (tid < REP * 64) L.qtab[tid / 64][tid % 64] = L.qraw[tid];   // raw fp16 rows: lane part = l%16 holds dims 8*part..+7
            if constexpr (REP == 1) iq_build_q<G, NWV>(L, tid, lane, a.scale_log2);
            if constexpr (REP > 1) {
                for (int i = tid; i < REP * NG; i += NT) {
                    float sq = 0.0f;
                    for (int d = 0; d < G; d++) sq += half_bits_to_float(qraw[(i / NG) * kD + (i % NG) * G + d]);
                    L.qsumg[i / NG][i % NG] = sq * kTwoM24;
                }
                for (int i = tid; i < AttnLds<G, REP, NWV>::WLS; i += NT) L.zrow[i] = 0;
                if (wave < 4) mc_build_q<G, REP>(L.qraw, lane, wave, L);
            }
            __syncthreads();
        };
        if constexpr (!kLateTables) { __syncthreads(); build_q_tables(); }

        WaveState<REP> st;
#pragma unroll
        for (int r = 0; r < REP; r++) {
            st.m[r] = -INFINITY; st.lsum[r] = 0.0f; st.z[r] = 0.0f; st.acc[r][0] = 0.0f; st.acc[r][1] = 0.0f;
#pragma unroll
            for (int ct = 0; ct < 8; ct++) st.accq[r][ct] = 0.0f;
        }
#pragma unroll
        for (int ct = 0; ct < 8; ct++) st.accA[ct] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
        float qp[4];

        // ---- (b) the row in segments whose chunk descriptors (block offset | log2 bits) sit in LDS.
        //      A ticket is one unit (<= 4 KiB of K codes + 4 KiB of V codes: 128/64/32/16 tokens at
        //      2/4/8/16 bits, or 16 rows of the FP16 residual), so every ticket costs about the same.
        //      The tickets of a segment are shared by all workgroups of the row through a counter in
        //      global memory: a workgroup is granted batches of consecutive tickets (guided sizes: a
        //      share of what is left, so the last batches are small and everybody finishes together)
        //      and its wavefronts draw from the granted range through a counter in LDS.
        for (int seg = 0; seg < n_seg; seg++) {
            const int cs = seg * seg_chunks, ce = min(C, cs + seg_chunks);
            if (seg > 0) __syncthreads();                // previous segment's tables consumed
            // chunks [cs + tid*KPT, +KPT) per thread: descriptor, units per chunk, exclusive scan
            uint32_t ucnt[2] = {0u, 0u}, mine = 0u;
#pragma unroll
            for (int k = 0; k < 2; k++) {
                const int c = cs + tid * KPT + k;
                if (k < KPT && c < ce) {
                    const int bits = bits_of(seg == 0 ? e_first[k] : erow[c]);
                    const int lgb = bits == 2 ? 1 : (bits == 4 ? 2 : (bits == 8 ? 3 : 4));
                    L.desc[c - cs] = (seg == 0 ? o_first[k] : orow[c]) | (unsigned long long)lgb;   // block offsets are multiples of 256
                    ucnt[k] = (uint32_t)((N + (256 >> lgb) - 1) >> (8 - lgb));
                    mine += ucnt[k];
                }
            }
            const uint32_t incl = wave_incl_scan(mine);
            if (lane == 63) L.wscan[wave] = incl;
            if (tid == 0) { L.next = (uint32_t)NWV; L.limit = 0; L.done = 0; L.fetching = 0; L.g_seen = 0; L.nb = 0; }   // the first draws are fixed: wavefront v holds local ticket v
            __syncthreads();
            uint32_t pos = incl - mine, n_chunk_units = 0;
#pragma unroll
            for (int wv = 0; wv < NWV; wv++) { if (wv < wave) pos += L.wscan[wv]; n_chunk_units += L.wscan[wv]; }
            const uint32_t T = n_chunk_units + (uint32_t)(seg == n_seg - 1 ? (n_tail + 15) / 16 : 0);
            unsigned int *counter = a.counters + ((size_t)u * n_seg + seg) * kCounterStride;
            // no cap for a workgroup whose whole interval lies in this row, or that covers the whole row
            const uint32_t quota = whole ? 0xffffffffu : (uint32_t)(((unsigned long long)T * ov + ru - 1) / ru);
            if (P == 1u) {                               // nobody shares the row: every ticket is this workgroup's, no counter in memory needed
                if (tid == 0) { L.bl[0] = 0u; L.bg[0] = 0u; L.nb = 1u; L.limit = T; L.g_seen = T; L.done = 1u; }
            } else if (seg == 0 && tid == 0) {           // the batch asked for during the row set-up
                const uint32_t granted = g_first < T ? min((uint32_t)NWV, T - g_first) : 0u;
                L.g_seen = g_first + (uint32_t)NWV;
                if (granted) { L.bl[0] = 0u; L.bg[0] = g_first; L.nb = 1u; L.limit = granted; }
                if (g_first + (uint32_t)NWV >= T || granted >= quota) L.done = 1u;
            }
#pragma unroll
            for (int k = 0; k < 2; k++) {
                const int c = cs + tid * KPT + k;
                if (k < KPT && c < ce) {
                    L.ustart[c - cs] = (uint16_t)pos;
                    for (uint32_t i = 0; i < ucnt[k]; i++) L.inv[pos + i] = (uint16_t)(c - cs);
                    pos += ucnt[k];
                }
            }
            __syncthreads();

            // One wavefront at a time asks the row's counter for the next batch.
            auto fetch = [&]() {
                if (lane == 0) {
                    const uint32_t limit = __atomic_load_n(&L.limit, __ATOMIC_RELAXED);
                    if (!__atomic_load_n(&L.done, __ATOMIC_RELAXED)) {
                        const uint32_t seen = L.g_seen, nb = L.nb;
                        // guided batch size from the counter value seen at the previous grant (none yet:
                        // the smallest batch), so that nobody sits on a large batch when the row runs dry
                        uint32_t want = (uint32_t)NWV;
                        if (nb > 0 && T > seen) want = max(want, (T - seen) / (4u * P));
                        if (nb >= (uint32_t)kMaxBatches - 1) want = T;                 // table full: all that is left
                        want = min(want, quota - limit);                               // limit < quota here
                        const uint32_t g0 = atomicAdd(counter, want);
                        L.g_seen = g0 + want;
                        uint32_t granted = 0;
                        if (g0 < T) {
                            granted = min(want, T - g0);
                            L.bl[nb] = limit; L.bg[nb] = g0; L.nb = nb + 1;
                            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                            __atomic_store_n(&L.limit, limit + granted, __ATOMIC_RELAXED);
                        }
                        if (g0 + want >= T || limit + granted >= quota) {
                            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                            __atomic_store_n(&L.done, 1u, __ATOMIC_RELAXED);
                        }
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                    __atomic_store_n(&L.fetching, 0u, __ATOMIC_RELAXED);
                }
            };
            auto try_fetch = [&]() -> bool {             // true if this wavefront held the lock (and fetched)
                uint32_t won = 0;
                if (lane == 0) won = atomicCAS(&L.fetching, 0u, 1u) == 0u ? 1u : 0u;
                won = (uint32_t)__builtin_amdgcn_readfirstlane((int)won);
                if (won) fetch();
                return won != 0;
            };

            // tickets: the draw for the next unit is issued when the current one is taken
            uint32_t pend = (uint32_t)wave;              // the first draw (L.next starts at NWV)
            int bcur = 0;                                // batch of this wavefront's latest ticket
            auto issue_draw = [&]() { if (lane == 0) pend = atomicAdd(&L.next, 1u); };
            auto next_unit = [&](Unit &un) -> bool {     // the pending draw becomes the next unit
                const uint32_t t = (uint32_t)__builtin_amdgcn_readfirstlane((int)pend);
                uint32_t limit;
                for (;;) {                               // wait until local ticket t is granted, or nothing is left
                    limit = (uint32_t)__builtin_amdgcn_readfirstlane((int)__atomic_load_n(&L.limit, __ATOMIC_RELAXED));
                    if (t < limit) break;
                    if (__builtin_amdgcn_readfirstlane((int)__atomic_load_n(&L.done, __ATOMIC_RELAXED))) {
                        limit = (uint32_t)__builtin_amdgcn_readfirstlane((int)__atomic_load_n(&L.limit, __ATOMIC_RELAXED));
                        if (t < limit) break;            // done is written after the last limit
                        return false;
                    }
                    if (!try_fetch()) __builtin_amdgcn_s_sleep(2);
                }
                if (t + (uint32_t)NWV >= limit && !__builtin_amdgcn_readfirstlane((int)__atomic_load_n(&L.done, __ATOMIC_RELAXED)))
                    try_fetch();                         // top up ahead of need; whoever gets the lock does it
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                while (bcur + 1 < __builtin_amdgcn_readfirstlane((int)__atomic_load_n(&L.nb, __ATOMIC_RELAXED)) &&
                       t >= (uint32_t)__builtin_amdgcn_readfirstlane((int)L.bl[bcur + 1])) bcur++;
                const uint32_t tk = (uint32_t)__builtin_amdgcn_readfirstlane((int)(L.bg[bcur] + (t - L.bl[bcur])));
                issue_draw();
                if (tk < n_chunk_units) {
                    const int cl = __builtin_amdgcn_readfirstlane((int)L.inv[tk]);
                    const unsigned long long dsc = L.desc[cl];
                    const uint32_t dlo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)dsc);
                    const uint32_t dhi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(dsc >> 32));
                    const int sidx = (int)tk - __builtin_amdgcn_readfirstlane((int)L.ustart[cl]);
                    const int lgb = (int)(dlo & 7u);
                    const uint8_t *blk = a.arena + (((unsigned long long)dhi << 32) | (dlo & ~0xffu));
                    const int t0 = sidx << (8 - lgb);
                    un.lgb = lgb;
                    un.nsub = max(min(4, (N - t0) >> (6 - lgb)), 1); un.nvalid = min(N - t0, 256 >> lgb); un.tail_rows = 1 << 20;
                    un.kb = blk; un.vb = blk;
                    if (lgb == 4) {
                        un.kc = (uint32_t)t0 << 8; un.vc = un.kc + ((uint32_t)N << 8);
                        un.km = un.kc; un.vm = un.kc;    // no meta: see load_k
                    } else {
                        const uint32_t cb = (uint32_t)N << (4 + lgb), mb = (uint32_t)N * NG * 4;
                        un.kc = (uint32_t)t0 << (4 + lgb);
                        un.km = KPC ? cb + (uint32_t)(t0 / G) * (kD * 4u) : cb + (uint32_t)t0 * NG * 4;
                        un.vc = un.kc + cb + mb;
                        un.vm = cb + mb + (SMALL ? (uint32_t)max(N, lgb == 1 ? 16 : 8) << (4 + lgb) : cb) + (uint32_t)t0 * NG * 4;   // 8 tokens at 2 bits: V codes of a whole slice
                    }
                } else {                                 // 16 rows of the FP16 residual
                    const int row0 = (int)(tk - n_chunk_units) * 16;
                    un.lgb = 4; un.nsub = SMALL ? min(4, N >> 2) : 4; un.nvalid = min(16, n_tail - row0); un.tail_rows = n_tail - row0;   // the buffers hold N rows
                    un.kb = reinterpret_cast<const uint8_t *>(a.K_tail) + (size_t)u * N * 256;
                    un.vb = reinterpret_cast<const uint8_t *>(a.V_tail) + (size_t)u * N * 256;
                    un.kc = un.vc = (uint32_t)row0 * 256u;
                    un.km = un.kc; un.vm = un.vc;
                }
                return true;
            };

            // K is requested half a unit ahead (right after the scores of the current unit), V a
            // whole unit ahead into the buffer the current unit does not use.
            Unit cur, nxt;
            KR kr;
            VRegs<G> va, vb;
            bool have = next_unit(cur);
            auto load_keys = [&](const Unit &un) {
                if constexpr (REP == 1) load_k_iq<G, KPC, SMALL>(un, lane, kr); else load_k_mc<G, REP, SMALL>(un, lane, kr);
            };
            if (have) { load_keys(cur); load_v<G, SMALL>(cur, lane, va, N); }
            if (seg == 0) {                              // the q tables, behind the first units' loads
                if constexpr (kLateTables) build_q_tables();
                if constexpr (REP > 1) {
                    const int slot0 = MC<G, REP>::slot0(lane >> 4);
#pragma unroll
                    for (int n = 0; n < 4; n++) qp[n] = L.qsumg[(slot0 + n) / NG][(slot0 + n) % NG];
                }
            }
            const float scale24 = a.scale_log2 * kTwo24;
            auto step = [&](const VRegs<G> &vc, VRegs<G> &vn) {
                const bool have_next = next_unit(nxt);
                const Unit &pf = have_next ? nxt : cur;  // nothing left: re-read the current unit (ignored)
                const int lgb = cur.lgb;
                float p4[REP][4];                         // fp16 units: weights handed from scores to values
                v4u ak[4];                                // grouped queries: the score operands of this bit-width
                if constexpr (REP > 1) {
                    const int bi = min(lgb, 3) - 1;
#pragma unroll
                    for (int mi = 0; mi < 4; mi++) ak[mi] = L.qmc[bi][mi][lane];
                }
                load_v<G, SMALL>(pf, lane, vn, N);              // a whole unit ahead
                if constexpr (REP == 1 && KPC) {
                    if (lgb == 1)      pc_scores<2, G, NWV>(cur, kr, lane, wave, a.scale_log2, L, st);
                    else if (lgb == 2) pc_scores<4, G, NWV>(cur, kr, lane, wave, a.scale_log2, L, st);
                    else if (lgb == 3) pc_scores<8, G, NWV>(cur, kr, lane, wave, a.scale_log2, L, st);
                    else                fp16_scores<G, REP, NWV>(cur, kr, lane, a.scale_log2, a.nq, a.rep_in, L, st, p4);
                    load_keys(pf);                        // half a unit ahead
                    if (lgb == 1)      iq_values<2, G, NWV>(vc, lane, wave, iq_weights<2, G, NWV>(vc, lane, wave, L, st), L, st);
                    else if (lgb == 2) iq_values<4, G, NWV>(vc, lane, wave, iq_weights<4, G, NWV>(vc, lane, wave, L, st), L, st);
                    else if (lgb == 3) iq_values<8, G, NWV>(vc, lane, wave, iq_weights<8, G, NWV>(vc, lane, wave, L, st), L, st);
                    else                fp16_values<G, REP, NWV>(cur, vc, lane, wave, L, st, p4);
                } else if constexpr (REP == 1) {
                    if (lgb == 1)      iq_scores<2, G, NWV, SMALL>(cur, kr, lane, wave, L, st);
                    else if (lgb == 2) iq_scores<4, G, NWV, SMALL>(cur, kr, lane, wave, L, st);
                    else if (lgb == 3) iq_scores<8, G, NWV, SMALL>(cur, kr, lane, wave, L, st);
                    else                fp16_scores<G, REP, NWV>(cur, kr, lane, a.scale_log2, a.nq, a.rep_in, L, st, p4);
                    load_keys(pf);                        // half a unit ahead
                    if (lgb == 1)      iq_values<2, G, NWV>(vc, lane, wave, iq_weights<2, G, NWV>(vc, lane, wave, L, st), L, st);
                    else if (lgb == 2) iq_values<4, G, NWV>(vc, lane, wave, iq_weights<4, G, NWV>(vc, lane, wave, L, st), L, st);
                    else if (lgb == 3) iq_values<8, G, NWV>(vc, lane, wave, iq_weights<8, G, NWV>(vc, lane, wave, L, st), L, st);
                    else                fp16_values<G, REP, NWV>(cur, vc, lane, wave, L, st, p4);
                } else {
                    if (lgb == 1)      mc_scores<2, G, REP, NWV>(cur, kr, ak, qp, lane, wave, scale24, L, st);
                    else if (lgb == 2) mc_scores<4, G, REP, NWV>(cur, kr, ak, qp, lane, wave, scale24, L, st);
                    else if (lgb == 3) mc_scores<8, G, REP, NWV>(cur, kr, ak, qp, lane, wave, scale24, L, st);
                    else                fp16_scores<G, REP, NWV>(cur, kr, lane, a.scale_log2, a.nq, a.rep_in, L, st, p4);
                    load_keys(pf);                        // half a unit ahead
                    if (lgb == 1)      value_weights<2, G, REP, NWV>(vc, lane, wave, L, st);
                    else if (lgb == 2) value_weights<4, G, REP, NWV>(vc, lane, wave, L, st);
                    else if (lgb == 3) value_weights<8, G, REP, NWV>(vc, lane, wave, L, st);
                    if (lgb == 1)      mc_value_dots<2, G, REP, NWV>(vc, lane, wave, L, st);
                    else if (lgb == 2) mc_value_dots<4, G, REP, NWV>(vc, lane, wave, L, st);
                    else if (lgb == 3) mc_value_dots<8, G, REP, NWV>(vc, lane, wave, L, st);
                    else                fp16_values<G, REP, NWV>(cur, vc, lane, wave, L, st, p4);
                }
                cur = nxt; have = have_next;
            };
            while (have) {
                step(va, vb);
                if (!have) break;
                step(vb, va);
            }
        }

        // ---- (c) fold the wavefronts' states: o[d] = acc[d] * 2^24 + sum_t p_t zero_{t,g(d)}
#pragma unroll
        for (int r = 0; r < REP; r++) {
            float lt = st.lsum[r], zt = st.z[r];
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) lt += __shfl_xor(lt, o);
#pragma unroll
            for (int o = 32; o >= NG; o >>= 1) zt += __shfl_xor(zt, o);   // lanes with equal lane % NG
            const float zg = __shfl(zt, (2 * lane) / G);
            float *dst = &L.comb[wave][r][0];
            dst[2 * lane] = fmaf(st.acc[r][0], kTwo24, zg);
            dst[2 * lane + 1] = fmaf(st.acc[r][1], kTwo24, zg);
            if (lane == 0) { dst[kD] = st.m[r]; dst[kD + 1] = lt; }
            if constexpr (REP == 1) {
                wave_sync();
#pragma unroll
                for (int ct = 0; ct < 8; ct++)            // column tile ct: the lane quarter of its group holds the sums
                    if ((lane >> 4) == (16 * ct) / G) dst[16 * ct + (lane & 15)] += st.accq[r][ct];
            }
        }
        if constexpr (REP > 1) {                          // matrix-core tiles: row = head * NG + group, column = dim
            wave_sync();
            const int x = lane & 15, qd = lane >> 4;
#pragma unroll
            for (int ct = 0; ct < 8; ct++) {
#pragma unroll
                for (int n = 0; n < 4; n++) {
                    const int slot = 4 * qd + n;
                    if (slot < REP * NG && slot % NG == (16 * ct) / G) {
                        float *dst = &L.comb[wave][slot / NG][16 * ct + x];
                        *dst = fmaf(st.accA[ct][n], kTwo24, *dst);
                    }
                }
            }
        }
        __syncthreads();
        const int slot = w - wg_first;
        for (int i = tid; i < REP * kD; i += NT) {
            const int r = i / kD, d = i % kD;
            float M = -INFINITY;
#pragma unroll
            for (int wv = 0; wv < NWV; wv++) M = fmaxf(M, L.comb[wv][r][kD]);
            float num = 0.0f, den = 0.0f;
#pragma unroll
            for (int wv = 0; wv < NWV; wv++) {
                const float f = (L.comb[wv][r][kD] == -INFINITY) ? 0.0f : fast_exp2(L.comb[wv][r][kD] - M);
                num = fmaf(L.comb[wv][r][d], f, num);
                den = fmaf(L.comb[wv][r][kD + 1], f, den);
            }
            float *dst = a.part + (((int64_t)u * REP + r) * a.max_partials + slot) * (kD + 2);
            dst[d] = num;
            if (d == 0) { dst[kD] = M; dst[kD + 1] = den; }
        }
    }
}

// Before the main kernel, one workgroup per row: zeroes the row's ticket counters (a kernel rather than a
// memset node, so that the call can be captured into a graph) and adds up the cost of the row's units.
__global__ __launch_bounds__(256) void attn_prep_kernel(AttnArgs a, int n_seg) {
    __shared__ uint32_t wsum[4];
    const int u = (int)blockIdx.x, tid = (int)threadIdx.x;
    for (int i = tid; i < n_seg; i += 256) a.counters[((size_t)u * n_seg + i) * kCounterStride] = 0u;
    uint32_t units = 0u;
    const uint8_t *erow = a.expert + (int64_t)u * a.desc_stride;
    const int NG = kD / a.G;
    int C = a.n_chunks, n_tail = a.n_tail;
    if (a.seq_chunks) {                                   // ragged batch: this row's own length
        C = min(max(a.seq_chunks[u / a.Hkv], 0), a.n_chunks);
        n_tail = min(max(a.seq_tail[u / a.Hkv], 0), a.N - 1);
    }
    for (int c = tid; c < C; c += 256) {                 // a unit costs its 8 KiB of codes plus its meta words, in steps of 512 bytes
        const int lgb = lgb_of_bits(bits_of_expert(a, erow[c]));
        units += units_of_chunk(a.N, lgb) * (uint32_t)(16 + (lgb < 4 ? (4 * NG) >> lgb : 0));
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) units += __shfl_xor(units, o);
    if ((tid & 63) == 0) wsum[tid >> 6] = units;
    __syncthreads();
    if (tid == 0) {
        // plus what the set-up of a row costs a workgroup (three round trips to memory and the tables: about as long
        // as 27 units take its eight wavefronts; 40 measured best), so that many short rows are not all handed to one workgroup
        const uint32_t units_cost = wsum[0] + wsum[1] + wsum[2] + wsum[3] + 16u * (uint32_t)((n_tail + 15) / 16);
        a.counters[(size_t)a.BH * n_seg * kCounterStride + u] = units_cost ? units_cost + kRowSetupCost : 0u;
        a.counters[(size_t)a.BH * n_seg * kCounterStride + a.BH + u] = 0u;   // workgroups of the row: stays 0 for a row without tokens
    }
}
int attn_row_segments(int n_chunks, int N) {
    const int sc = attn_segment_chunks(N);
    return n_chunks > sc ? (n_chunks + sc - 1) / sc : 1;
}
size_t attn_counter_bytes(int BH, int n_chunks, int N) {
    // ticket counters, then the rows' unit counts and workgroup counts
    return ((size_t)BH * attn_row_segments(n_chunks, N) * kCounterStride + 2 * (size_t)BH) * sizeof(unsigned int);
}

// out[b, hq, :] = sum_p o_p 2^(m_p - M) / sum_p l_p 2^(m_p - M) over the partials of the row
// (one per workgroup that touched the row's KV head).  Thread (grp, d) takes the partials grp, grp + 8, ...:
// with the usual 6-8 partials per row every value is requested at once, one round trip to memory.
constexpr int kMergeGroups = 8;
__global__ __launch_bounds__(kD *kMergeGroups) void attn_merge_kernel(const float *__restrict__ part,
                                                                       float *__restrict__ out, int rep,
                                                                       const uint32_t *__restrict__ row_wgs, int max_partials,
                                                                       unsigned int *zero_counters, int n_seg, int Hkv, int nq, int rep_in) {
    __shared__ float numl[kMergeGroups][kD];
    __shared__ float denl[kMergeGroups], ml[kMergeGroups];
    const int row = (int)blockIdx.x, tid = (int)threadIdx.x, d = tid & (kD - 1), grp = tid >> 7;
    const int u = row / rep;
    // calls that run on a plan (moqae_decode_plan) leave the ticket counters as they found them: zero
    if (zero_counters && row % rep == 0)
        for (int i = tid; i < n_seg; i += kD * kMergeGroups) zero_counters[((size_t)u * n_seg + i) * kCounterStride] = 0u;
    const int P = (int)row_wgs[u];
    const float *p0 = part + (int64_t)row * max_partials * (kD + 2);
    // this group's partials, merged on the way (online rescaling)
    float m = -INFINITY, num = 0.0f, den = 0.0f;
    for (int p = grp; p < P; p += kMergeGroups) {
        const float *pp = p0 + (int64_t)p * (kD + 2);
        const float mp = pp[kD], lp = pp[kD + 1], op = pp[d];
        const float mn = fmaxf(m, mp);
        const float fo = (m == -INFINITY) ? 0.0f : fast_exp2(m - mn), fp = (mp == -INFINITY) ? 0.0f : fast_exp2(mp - mn);   // empty partials
        num = fmaf(num, fo, op * fp);
        den = fmaf(den, fo, lp * fp);
        m = mn;
    }
    numl[grp][d] = num;
    if (d == 0) { denl[grp] = den; ml[grp] = m; }
    __syncthreads();
    if (grp == 0) {
        float M = -INFINITY;
#pragma unroll
        for (int g = 0; g < kMergeGroups; g++) M = fmaxf(M, ml[g]);
        float n = 0.0f, dn = 0.0f;
#pragma unroll
        for (int g = 0; g < kMergeGroups; g++) {
            const float f = (ml[g] == -INFINITY) ? 0.0f : fast_exp2(ml[g] - M);
            n = fmaf(numl[g][d], f, n); dn = fmaf(denl[g], f, dn);
        }
        const int rr = row % rep;                                       // out [B, nq, Hkv * rep_in, D]: head rr = query rr / rep_in
        const int64_t orow = ((int64_t)(u / Hkv) * nq + rr / rep_in) * (Hkv * rep_in) + (u % Hkv) * rep_in + rr % rep_in;
        out[orow * kD + d] = dn > 0.0f ? n / dn : 0.0f;                 // a sequence without tokens: zeros
    }
}

template <int REP> constexpr int waves_per_wg() { return 8; }

// The split kernel of a call: the instantiation for its batch shape (uniform / ragged) and chunk size.
template <int G, int REP, bool KPC>
static void launch_split(const AttnArgs &a, dim3 grid, dim3 block, hipStream_t s) {
    constexpr int NWV = waves_per_wg<REP>();
    if (a.N < 64) {
        if (a.seq_chunks) hipLaunchKernelGGL((attn_split_kernel<G, REP, NWV, true, true, KPC>), grid, block, 0, s, a);
        else              hipLaunchKernelGGL((attn_split_kernel<G, REP, NWV, false, true, KPC>), grid, block, 0, s, a);
    } else {
        if (a.seq_chunks) hipLaunchKernelGGL((attn_split_kernel<G, REP, NWV, true, false, KPC>), grid, block, 0, s, a);
        else              hipLaunchKernelGGL((attn_split_kernel<G, REP, NWV, false, false, KPC>), grid, block, 0, s, a);
    }
}

template <int G, int REP>
static hipError_t launch_gr(const AttnArgs &a, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end) {
    constexpr int NWV = waves_per_wg<REP>();
    const int n_seg = attn_row_segments(a.n_chunks, a.N);
    if (a.kpc && REP != 1) return hipErrorInvalidValue;  // per-channel keys: one query head per KV head (checked by the caller)
    if (!a.planned) {
        hipLaunchKernelGGL(attn_prep_kernel, dim3((unsigned)a.BH), dim3(256), 0, s, a, n_seg);
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
    }
    if (ev_begin && hipEventRecord(ev_begin, s) != hipSuccess) return hipErrorInvalidValue;
    const dim3 grid((unsigned)a.n_wg), block(NWV * 64);
    if constexpr (REP == 1) {
        if (a.kpc) launch_split<G, REP, true>(a, grid, block, s);
        else       launch_split<G, REP, false>(a, grid, block, s);
    } else {
        launch_split<G, REP, false>(a, grid, block, s);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ev_end && hipEventRecord(ev_end, s) != hipSuccess) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_merge_kernel, dim3((unsigned)(a.BH * a.rep)), dim3(kD * kMergeGroups), 0, s,
                       (const float *)a.part, a.out, a.rep,
                       (const uint32_t *)(a.counters + (size_t)a.BH * n_seg * kCounterStride + a.BH), a.max_partials,
                       a.planned ? a.counters : (unsigned int *)nullptr, n_seg, a.Hkv, a.nq, a.rep_in);
    return hipGetLastError();
}

#define MOQAE_FOR_EACH_VARIANT(X) X(64, 1) X(64, 2) X(64, 4) X(64, 8) X(32, 1) X(32, 2) X(32, 4)

int attn_waves_per_wg(int rep) { (void)rep; return 8; }

// The first kernel of a decode call alone: ticket counters zeroed, the rows' costs (with a nominal residual of half
// a chunk, so that a row with any token has a cost) and zero workgroup counts left in the workspace.
hipError_t launch_attn_plan(const AttnArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(attn_prep_kernel, dim3((unsigned)a.BH), dim3(256), 0, s, a, attn_row_segments(a.n_chunks, a.N));
    return hipGetLastError();
}

hipError_t launch_attn(const AttnArgs &a, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end) {
#define MOQAE_CASE(GV, RV) if (a.G == GV && a.rep == RV) return launch_gr<GV, RV>(a, s, ev_begin, ev_end);
    MOQAE_FOR_EACH_VARIANT(MOQAE_CASE)
#undef MOQAE_CASE
    return hipErrorInvalidValue;
}

}  // namespace moqae
