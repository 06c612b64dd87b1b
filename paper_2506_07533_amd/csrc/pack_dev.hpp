// Device code of the quantiser / packer shared by pack_kernel and the fused route + pack kernel.
#pragma once
#include "moqae_dev.hpp"

namespace moqae {

// The packed cache is written once and read much later by another kernel: streaming stores keep it
// from displacing (and later being written back from under) what the caches hold.
template <typename T> __device__ __forceinline__ void nt_store(T *p, T v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void nt_store(uint4 *p, uint4 v) {
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store(u4{v.x, v.y, v.z, v.w}, reinterpret_cast<u4 *>(p));
}
__device__ __forceinline__ void nt_store(uint2 *p, uint2 v) {
    typedef uint32_t u2 __attribute__((ext_vector_type(2)));
    __builtin_nontemporal_store(u2{v.x, v.y}, reinterpret_cast<u2 *>(p));
}

__device__ __forceinline__ uint4 nt_load(const uint4 *p) {
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    const u4 v = __builtin_nontemporal_load(reinterpret_cast<const u4 *>(p));
    return uint4{v[0], v[1], v[2], v[3]};
}

constexpr int kPackThreads = 256;
constexpr int kVRow = kD + 4;                        // bytes per token row of the V staging buffer

// Position of the code with in-word index e (b bits): even e in the low half-word, odd e high.
__device__ __forceinline__ constexpr int code_shift(int e, int b) { return 16 * (e & 1) + b * (e >> 1); }

// Element-wise minimum / maximum of two fp16 pairs (finite inputs).
__device__ __forceinline__ uint32_t pk_min_f16(uint32_t x, uint32_t y) {
    uint32_t r;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
    return r;
}
__device__ __forceinline__ uint32_t pk_max_f16(uint32_t x, uint32_t y) {
    uint32_t r;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
    return r;
}
// binary32 sum of one fp16 half of w and c, rounded once: the conversion of the half is exact and rides
// along in the mixed-precision multiply-add (x * 1 + c), so this is the binary32 subtraction x - (-c).
__device__ __forceinline__ float add_lo_f16(uint32_t w, float c) {
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel_hi:[1,0,0]" : "=v"(r) : "v"(w), "v"(c));
    return r;
}
__device__ __forceinline__ float add_hi_f16(uint32_t w, float c) {
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(w), "v"(c));
    return r;
}

// rint(t) for 0 <= t < 2^22 without a conversion: t + 1.5 * 2^23 is rounded to an integer by the addition
// itself (ties to even), and the integer sits in the low mantissa bits: bits(result) = kMagicBits + rint(t).
constexpr float kMagic = 12582912.0f;
constexpr uint32_t kMagicBits = 0x4B400000u;

// One (token row, group) item of a quantised chunk: G consecutive dims, all in one lane.  No lane ever
// needs another lane's data: minimum and maximum come from packed fp16 operations on the words as
// loaded, scale and reciprocal are computed once per group, and a code costs four operations: x - min
// (with the conversion folded in), * 1/scale, + magic (the rounding), shift-and-add into its word.  The
// words are sums of bits(t + magic) << shift, i.e. of the codes plus a constant that is taken off at
// the end; no code is ever masked.  No clamp is needed: the scale is rounded up, so that
// (x - min) * (1/scale) <= qmax * (1 + 2e-7) and rounds to at most qmax, and x >= min.
// STAGED: meta_dst is a register of the caller and k_dst a staging row in LDS (plain stores), see pack_row.
template <int G, int BITS, bool STAGED = false>
__device__ __forceinline__ void pack_item_regs(const uint32_t *w, bool isV, uint32_t *__restrict__ meta_dst,
                                               uint32_t *__restrict__ k_dst, uint32_t *__restrict__ v_lds) {
    constexpr int NW = G / 2;                        // input words (fp16 pairs) of the item, w[0..NW)
    static_assert(NW >= 16, "G >= 32");
    uint32_t mn4[4], mx4[4];                          // four independent chains, folded at the end
#pragma unroll
    for (int k = 0; k < 4; k++) { mn4[k] = pk_min_f16(w[k], w[k + 4]); mx4[k] = pk_max_f16(w[k], w[k + 4]); }
#pragma unroll
    for (int k = 8; k < NW; k++) { mn4[k & 3] = pk_min_f16(mn4[k & 3], w[k]); mx4[k & 3] = pk_max_f16(mx4[k & 3], w[k]); }
    const uint32_t mnp = pk_min_f16(pk_min_f16(mn4[0], mn4[1]), pk_min_f16(mn4[2], mn4[3]));
    const uint32_t mxp = pk_max_f16(pk_max_f16(mx4[0], mx4[1]), pk_max_f16(mx4[2], mx4[3]));
    float mn = fminf(half_bits_to_float(mnp & 0xffffu), half_bits_to_float(mnp >> 16));
    float mx = fmaxf(half_bits_to_float(mxp & 0xffffu), half_bits_to_float(mxp >> 16));
    if (mn == 0.0f) mn = 0.0f;                        // -0 is stored as +0
    if (mx == 0.0f) mx = 0.0f;
    constexpr float qmax = (float)((1 << BITS) - 1);
    const float R = __fsub_rn(mx, mn);
    const float s32 = __fdiv_rn(R, qmax);
    uint32_t s16 = float_to_half_bits(s32);
    if (half_bits_to_float(s16) < s32) s16 += 1;      // the scale is rounded up
    if (s16 == 0) s16 = 0x3C00u;                      // constant group: scale 1
    const float inv = __fdiv_rn(1.0f, half_bits_to_float(s16));
    if constexpr (STAGED) *meta_dst = s16 | (float_to_half_bits(mn) << 16);
    else                  nt_store(meta_dst, s16 | (float_to_half_bits(mn) << 16));
    const float nmn = -mn;
    auto ubits = [&](int d) -> uint32_t {             // kMagicBits + code of dim d of the item
        const float diff = (d & 1) ? add_hi_f16(w[d >> 1], nmn) : add_lo_f16(w[d >> 1], nmn);
        return __builtin_bit_cast(uint32_t, __fadd_rn(__fmul_rn(diff, inv), kMagic));
    };
    if (isV) {                                        // one code per byte into the staging rows
        constexpr uint32_t KC = kMagicBits * 0x01010101u;
#pragma unroll
        for (int k = 0; k < G / 4; k++) {
            uint32_t acc = ubits(4 * k);
            acc += ubits(4 * k + 1) << 8; acc += ubits(4 * k + 2) << 16; acc += ubits(4 * k + 3) << 24;
            v_lds[k] = acc - KC;
        }
    } else {                                          // the words of the token-major K layout
        constexpr int CPW = 32 / BITS, WPL = G / CPW;
        uint32_t ksum = 0;
#pragma unroll
        for (int e = 0; e < CPW; e++) ksum += 1u << code_shift(e, BITS);
        const uint32_t KC = kMagicBits * ksum;        // constant folded (wraps like the sums do)
        uint32_t out[WPL];
#pragma unroll
        for (int k = 0; k < WPL; k++) {
            uint32_t acc = ubits(k * CPW);
#pragma unroll
            for (int e = 1; e < CPW; e++) acc += ubits(k * CPW + e) << code_shift(e, BITS);
            out[k] = acc - KC;
        }
        if constexpr (WPL >= 4) {
#pragma unroll
            for (int k = 0; k < WPL; k += 4) {
                const uint4 o = uint4{out[k], out[k + 1], out[k + 2], out[k + 3]};
                if constexpr (STAGED) *reinterpret_cast<uint4 *>(k_dst + k) = o;
                else                  nt_store(reinterpret_cast<uint4 *>(k_dst + k), o);
            }
        } else {
            static_assert(WPL == 2, "G = 32 at 2 bits");
            if constexpr (STAGED) *reinterpret_cast<uint2 *>(k_dst) = uint2{out[0], out[1]};
            else                  nt_store(reinterpret_cast<uint2 *>(k_dst), uint2{out[0], out[1]});
        }
    }
}

// The same from memory: p = the item's G fp16 values.
template <int G, int BITS>
__device__ __forceinline__ void pack_item(const uint4 *__restrict__ p, bool isV, uint32_t *__restrict__ meta_dst,
                                          uint32_t *__restrict__ k_dst, uint32_t *__restrict__ v_lds) {
    uint32_t w[G / 2];
#pragma unroll
    for (int j = 0; j < G / 8; j++) {                // the whole item is requested at once: its 128-byte line arrives once
        // (ordinary loads: the lane's eight loads share the line through the cache; streaming loads here fetch it eight times)
        const uint4 t = p[j];
        w[4 * j] = t.x; w[4 * j + 1] = t.y; w[4 * j + 2] = t.z; w[4 * j + 3] = t.w;
    }
    pack_item_regs<G, BITS>(w, isV, meta_dst, k_dst, v_lds);
}

// Keys quantised per channel: a group is G consecutive tokens of one dim.  One wavefront per token group, lane l owns
// dims 2l, 2l+1 (one 32-bit column of fp16 pairs): it reads the G rows' words (a row is one coalesced 256-byte piece per
// wavefront), takes the packed minimum / maximum over the tokens, computes scale and reciprocal of both dims as
// pack_item does (the same binary32 operations, so the same bits), then per token its two codes, which the n/2
// lanes of a code word OR together (DPP) before one of them stores the word at its token-major place.
template <int G, int BITS>
__device__ __forceinline__ void pack_k_channel_group(const uint16_t *src, int64_t stride_s, int tg, uint32_t *codes_w,
                                                     uint32_t *meta_w, int lane) {
    const uint32_t *col = reinterpret_cast<const uint32_t *>(src + (int64_t)tg * G * stride_s) + lane;
    const int64_t rw = stride_s / 2;                  // row stride in words
    uint32_t w[G];
#pragma unroll
    for (int i = 0; i < G; i++) w[i] = col[i * rw];
    uint32_t mn4[4], mx4[4];
#pragma unroll
    for (int k = 0; k < 4; k++) { mn4[k] = pk_min_f16(w[k], w[k + 4]); mx4[k] = pk_max_f16(w[k], w[k + 4]); }
#pragma unroll
    for (int k = 8; k < G; k++) { mn4[k & 3] = pk_min_f16(mn4[k & 3], w[k]); mx4[k & 3] = pk_max_f16(mx4[k & 3], w[k]); }
    const uint32_t mnp = pk_min_f16(pk_min_f16(mn4[0], mn4[1]), pk_min_f16(mn4[2], mn4[3]));
    const uint32_t mxp = pk_max_f16(pk_max_f16(mx4[0], mx4[1]), pk_max_f16(mx4[2], mx4[3]));
    constexpr float qmax = (float)((1 << BITS) - 1);
    float nmn[2], inv[2];
    uint32_t metaw[2];
#pragma unroll
    for (int e = 0; e < 2; e++) {
        float mn = half_bits_to_float((mnp >> (16 * e)) & 0xffffu), mx = half_bits_to_float((mxp >> (16 * e)) & 0xffffu);
        if (mn == 0.0f) mn = 0.0f;                    // -0 is stored as +0
        if (mx == 0.0f) mx = 0.0f;
        const float s32 = __fdiv_rn(__fsub_rn(mx, mn), qmax);
        uint32_t s16 = float_to_half_bits(s32);
        if (half_bits_to_float(s16) < s32) s16 += 1;  // the scale is rounded up
        if (s16 == 0) s16 = 0x3C00u;                  // constant group: scale 1
        inv[e] = __fdiv_rn(1.0f, half_bits_to_float(s16));
        nmn[e] = -mn;
        metaw[e] = s16 | (float_to_half_bits(mn) << 16);
    }
    nt_store(reinterpret_cast<uint2 *>(meta_w + (size_t)tg * kD + 2 * lane), uint2{metaw[0], metaw[1]});
    constexpr int CPW = 32 / BITS, LPW = CPW / 2;     // codes per word, lanes per word
    const int pi = lane % LPW;                        // this lane's pair inside its word
    uint32_t *dst = codes_w + (size_t)tg * G * (kD / CPW) + lane / LPW;
#pragma unroll
    for (int i = 0; i < G; i++) {
        const uint32_t c0 = __builtin_bit_cast(uint32_t, __fadd_rn(__fmul_rn(add_lo_f16(w[i], nmn[0]), inv[0]), kMagic)) - kMagicBits;
        const uint32_t c1 = __builtin_bit_cast(uint32_t, __fadd_rn(__fmul_rn(add_hi_f16(w[i], nmn[1]), inv[1]), kMagic)) - kMagicBits;
        uint32_t x = (c0 << (BITS * pi)) | (c1 << (16 + BITS * pi));
        x |= dpp_u<DPP_XOR1>(x);
        if constexpr (LPW >= 4) x |= dpp_u<DPP_XOR2>(x);
        if constexpr (LPW >= 8) x |= dpp_u<DPP_HALF_MIRROR>(x);
        if (pi == 0) nt_store(dst + (size_t)i * (kD / CPW), x);
    }
}

// The V codes of a chunk from the staging rows (vcodes: one code per byte, kVRow bytes per token row) into the
// dimension-major tile layout at codes_w, by NT threads; room = v_token_room(N, bits).
// V: dimension-major tiles of 16*QD slots x 4 words.  A slot holds TQ = max(TW, 8) consecutive tokens
// (TW = 32/bits per word, WD = TQ/TW words) of CPK = 4/WD dimensions that lie 16 apart; a token block is
// TB = min(4*TQ, room) tokens = QD slices (QD = 4, i.e. 1-KiB tiles, for N >= 64; a shorter chunk is one block of
// 1, 2 or 4 slices; 8 tokens at 2 bits fill half a slice); slot 16*qd + j of tile cg of a block: dims
// 16*(cg*CPK + n/WD) + j, token slice qd.
template <int BITS>
__device__ __forceinline__ void v_gather_bits(int N, int room, uint32_t *codes_w, const uint8_t *vcodes, int tid, int NT) {
    constexpr int TW = 32 / BITS, TQ = TW > 8 ? TW : 8, WD = TQ / TW, CPK = 4 / WD, NCG = kD / (16 * CPK);
    const int TB = min(4 * TQ, room), QD = TB / TQ;
    const int n_groups = room * kD * BITS / 128;      // a thread builds the words of four adjacent dims at a time
    for (int g = tid; g < n_groups; g += NT) {
        const int n = g & 3, jq = (g >> 2) & 3, qd = (g >> 4) & (QD - 1), tile = g / (16 * QD);
        const int cg = tile % NCG, block = tile / NCG;
        const int d0 = 16 * (cg * CPK + n / WD) + 4 * jq, t0 = block * TB + qd * TQ + (n % WD) * TW;
        uint32_t wk[4] = {0u, 0u, 0u, 0u};
        const uint8_t *src = vcodes + t0 * kVRow + d0;                  // the codes of dims d0..d0+3 of token t0 + e: word e*kVRow
        if (t0 + TW <= N) {
            // tokens 2k (low half-word) and 2k+1 (high) of a word share the shift BITS*k: one byte permute puts the two
            // codes of a dim in place, one shift-or adds the pair to the dim's word
#pragma unroll
            for (int k = 0; k < TW / 2; k++) {
                const uint32_t ev = *reinterpret_cast<const uint32_t *>(src + (2 * k) * kVRow);
                const uint32_t od = *reinterpret_cast<const uint32_t *>(src + (2 * k + 1) * kVRow);
#pragma unroll
                for (int j = 0; j < 4; j++)           // bytes 0..3 of the selector's source are `ev`, 4..7 `od`; 0x0c gives zero
                    wk[j] |= __builtin_amdgcn_perm(od, ev, 0x0c000c00u | (uint32_t)j | ((uint32_t)(4 + j) << 16)) << (BITS * k);
            }
        } else {                                      // tokens past the chunk (half a slice): zero codes
            const int te = min(TW, N - t0);
            for (int e = 0; e < te; e++) {
                const uint32_t v4 = *reinterpret_cast<const uint32_t *>(src + e * kVRow);
                const int sh = code_shift(e, BITS);
                wk[0] |= (v4 & 0xffu) << sh; wk[1] |= ((v4 >> 8) & 0xffu) << sh; wk[2] |= ((v4 >> 16) & 0xffu) << sh; wk[3] |= (v4 >> 24) << sh;
            }
        }
        // thread n = 0..3 of a quad holds word n of the slots 16*qd + 4*jq + k, k = 0..3: a 4 x 4 transpose inside
        // the quad leaves every thread with one whole slot, stored with one 16-byte store
#pragma unroll
        for (int k = 0; k < 4; k += 2) {
            const uint32_t r = dpp_u<DPP_XOR1>((n & 1) ? wk[k] : wk[k + 1]);
            if (n & 1) wk[k] = r; else wk[k + 1] = r;
        }
#pragma unroll
        for (int k = 0; k < 2; k++) {
            const uint32_t r = dpp_u<DPP_XOR2>((n & 2) ? wk[k] : wk[k + 2]);
            if (n & 2) wk[k] = r; else wk[k + 2] = r;
        }
        nt_store(reinterpret_cast<uint4 *>(codes_w + (tile * 16 * QD + 16 * qd + 4 * jq + n) * 4), uint4{wk[0], wk[1], wk[2], wk[3]});
    }
}
__device__ __forceinline__ void v_gather(int N, int bits, int room, uint32_t *codes_w, const uint8_t *vcodes, int tid, int NT) {
    if (bits == 2)      v_gather_bits<2>(N, room, codes_w, vcodes, tid, NT);
    else if (bits == 4) v_gather_bits<4>(N, room, codes_w, vcodes, tid, NT);
    else                v_gather_bits<8>(N, room, codes_w, vcodes, tid, NT);
}

// Token rows of a chunk from memory into the registers of the threads that own them (thread 64*wave + lane: row
// 64*wave + lane), in two steps.  A lane that reads its own row alone touches lines nobody else in the wavefront
// touches, sixteen times over: a read-only kernel of that shape moves 4.9 TB/s on this chip, one of whole lines per
// group of eight lanes 7.0 TB/s.  rows_request: load instruction 8h + j reads the half rows h of rows 8j .. 8j+7 of the
// wavefront, lane l the 16-byte piece l%8 of row 8j + l/8 (streaming loads: nothing is read twice).
// rows_transpose: through a buffer of 64 rows of kTRow bytes per wavefront in LDS (tbuf: the workgroup's buffers),
// half a row at a time, every lane takes the sixteen pieces of its own row.  Rows past the chunk's N read row N - 1.
constexpr int kTRow = 128 + 16;                      // + 16: the rows start on different banks
__device__ __forceinline__ void rows_request(const uint16_t *chunk, int64_t stride_s, int N, int wave, int lane, uint4 (&v)[16]) {
    const int r8 = lane >> 3, p = lane & 7;
#pragma unroll
    for (int h = 0; h < 2; h++) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int row = min(wave * 64 + 8 * j + r8, N - 1);
            v[8 * h + j] = nt_load(reinterpret_cast<const uint4 *>(chunk + (int64_t)row * stride_s + h * 64) + p);
        }
    }
}
__device__ __forceinline__ void wave_lds_sync() {     // orders a wavefront's own LDS traffic between two phases
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}
__device__ __forceinline__ void rows_transpose(const uint4 (&v)[16], uint8_t *tbuf, int wave, int lane, uint4 (&x)[16]) {
    const int r8 = lane >> 3, p = lane & 7;
    uint8_t *mine = tbuf + wave * (64 * kTRow);
#pragma unroll
    for (int h = 0; h < 2; h++) {
#pragma unroll
        for (int j = 0; j < 8; j++) *reinterpret_cast<uint4 *>(mine + (8 * j + r8) * kTRow + p * 16) = v[8 * h + j];
        wave_lds_sync();
#pragma unroll
        for (int k = 0; k < 8; k++) x[8 * h + k] = *reinterpret_cast<const uint4 *>(mine + lane * kTRow + k * 16);
        wave_lds_sync();
    }
}

// One token row (sixteen 16-byte pieces, in registers) of a chunk's K (isV = 0) or V (isV = 1) -> the chunk's block at
// bit-width `bits`: its NG items as pack_side would pack them, by the thread that owns the row.  Consecutive lanes own
// consecutive rows, so what a lane would store itself are pieces of lines: the row's meta words leave as one
// store per lane (a contiguous run over the wavefront), the K codes go to staging rows in LDS (`stage`, kKStageRow(bits)
// bytes per row) from where k_flush writes them out in whole lines, the V codes to the staging rows of v_gather.
__host__ __device__ __forceinline__ constexpr int k_stage_row(int bits) { return kD * bits / 8 + 16; }   // + 16: rows start on different banks
template <int G>
__device__ __forceinline__ void pack_row(const uint4 (&x)[16], int row, int N, int bits, int isV, uint8_t *blk, uint8_t *stage) {
    if (bits == 16) {                                 // FP16 expert: the row copied verbatim (through the cache: it merges the pieces)
        uint4 *dst = reinterpret_cast<uint4 *>(blk + (isV ? (size_t)N * kD * 2 : 0)) + row * 16;
#pragma unroll
        for (int j = 0; j < 16; j++) dst[j] = x[j];
        return;
    }
    constexpr int NG = kD / G, NW = G / 2;
    const int room = isV ? v_token_room(N, bits) : N;
    const size_t k_code_bytes = (size_t)N * kD * bits / 8, meta_bytes = (size_t)N * NG * 4;
    uint8_t *area = blk + (isV ? k_code_bytes + meta_bytes : 0);
    uint32_t *meta_w = reinterpret_cast<uint32_t *>(area + (size_t)room * kD * bits / 8);
    uint32_t w[kD / 2], mw[NG];
#pragma unroll
    for (int j = 0; j < 16; j++) { w[4 * j] = x[j].x; w[4 * j + 1] = x[j].y; w[4 * j + 2] = x[j].z; w[4 * j + 3] = x[j].w; }
#pragma unroll
    for (int g = 0; g < NG; g++) {
        uint32_t *vl = reinterpret_cast<uint32_t *>(stage + row * kVRow + g * G);
        uint32_t *kl = reinterpret_cast<uint32_t *>(stage + row * k_stage_row(bits) + g * (G * bits / 8));
        if (bits == 2)      pack_item_regs<G, 2, true>(&w[g * NW], isV, &mw[g], kl, vl);
        else if (bits == 4) pack_item_regs<G, 4, true>(&w[g * NW], isV, &mw[g], kl, vl);
        else                pack_item_regs<G, 8, true>(&w[g * NW], isV, &mw[g], kl, vl);
    }
    if constexpr (NG == 2) nt_store(reinterpret_cast<uint2 *>(meta_w + row * NG), uint2{mw[0], mw[1]});
    else                   nt_store(reinterpret_cast<uint4 *>(meta_w + row * NG), uint4{mw[0], mw[1], mw[2], mw[3]});
}

// The K codes of a chunk from the staging rows of pack_row to their token-major place, 16 bytes per thread and step.
__device__ __forceinline__ void k_flush(int N, int bits, uint8_t *blk, const uint8_t *stage, int tid, int NT) {
    const int ppr = kD * bits / 128, srow = k_stage_row(bits);     // 16-byte pieces per row: 2, 4, 8
    uint4 *dst = reinterpret_cast<uint4 *>(blk);
    for (int p = tid; p < N * ppr; p += NT) {
        const int row = p / ppr, col = p % ppr;
        nt_store(&dst[p], *reinterpret_cast<const uint4 *>(stage + row * srow + col * 16));
    }
}

// K (isV = 0) or V (isV = 1) of one chunk -> its block `blk` at bit-width `bits`, by one workgroup of NT threads
// (a multiple of 64).  src: the chunk's first row (row stride stride_s elements); vcodes: N * kVRow bytes of LDS (V only).
// KPC: the keys' groups run along tokens (pack_k_channel_group); a template flag so that its G registers per lane stay out
// of the ordinary kernels.
template <int G, bool KPC>
__device__ __forceinline__ void pack_side(const uint16_t *src, int64_t stride_s, int N, int bits, int isV, uint8_t *blk,
                                          uint8_t *vcodes, int tid, int NT = kPackThreads) {
    if (bits == 16) {                                 // FP16 expert: rows copied verbatim
        const int lane16 = tid & 15, rsub = tid >> 4;
        uint4 *dst = reinterpret_cast<uint4 *>(blk + (isV ? (size_t)N * kD * 2 : 0));
        for (int row = rsub; row < N; row += NT / 16)
            nt_store(&dst[row * 16 + lane16], nt_load(reinterpret_cast<const uint4 *>(src + (int64_t)row * stride_s + lane16 * 8)));
        return;
    }

    constexpr int NG = kD / G;                        // groups per row
    const int room = isV ? v_token_room(N, bits) : N;  // tokens the code area has room for (V: at least one slice)
    const size_t k_code_bytes = (size_t)N * kD * bits / 8, meta_bytes = (size_t)N * NG * 4;
    uint8_t *area = blk + (isV ? k_code_bytes + meta_bytes : 0);
    uint32_t *codes_w = reinterpret_cast<uint32_t *>(area);
    uint32_t *meta_w = reinterpret_cast<uint32_t *>(area + (size_t)room * kD * bits / 8);

    if (KPC && !isV) {                               // keys quantised per channel: one wavefront per group of G tokens
        for (int tg = tid >> 6; tg < N / G; tg += NT >> 6) {
            if (bits == 2)      pack_k_channel_group<G, 2>(src, stride_s, tg, codes_w, meta_w, tid & 63);
            else if (bits == 4) pack_k_channel_group<G, 4>(src, stride_s, tg, codes_w, meta_w, tid & 63);
            else                pack_k_channel_group<G, 8>(src, stride_s, tg, codes_w, meta_w, tid & 63);
        }
        return;
    }
    // item = (token row, group): consecutive lanes take consecutive 2G-byte pieces of the chunk
    for (int item = tid; item < N * NG; item += NT) {
        const int row = item / NG, g = item % NG;
        const uint4 *p = reinterpret_cast<const uint4 *>(src + (int64_t)row * stride_s + g * G);
        uint32_t *vl = reinterpret_cast<uint32_t *>(vcodes + row * kVRow + g * G);
        if (bits == 2)      pack_item<G, 2>(p, isV, &meta_w[item], codes_w + item * (G / 16), vl);
        else if (bits == 4) pack_item<G, 4>(p, isV, &meta_w[item], codes_w + item * (G / 8), vl);
        else                pack_item<G, 8>(p, isV, &meta_w[item], codes_w + item * (G / 4), vl);
    }
    if (!isV) return;

    __syncthreads();
    v_gather(N, bits, room, codes_w, vcodes, tid, NT);
}

}  // namespace moqae
