// moqae_quantize_pack: offset plan + group-wise quantisation and bit-packing of every chunk
// at its routed bit-width (Sec. 3.1-3.2 of the paper say only that a chunk is quantised with
// the configuration its router chose; the quantiser and the layout are defined in moqae.h).
//
//   plan_rows_kernel / plan_kernel  block sizes -> exclusive scan in (b, h, c) order -> offsets and
//                capacity check: one workgroup per row when the table allows, else one workgroup.
//   pack_kernel  one workgroup per (K or V, chunk, row), one lane per (token row, group): the lane loads its
//                G dims, takes minimum and maximum with packed fp16 operations, computes scale and
//                reciprocal once and then four operations per code (no cross-lane step anywhere).
//                K words are assembled in registers (row-major layout); V codes go through LDS as
//                bytes and are gathered token-wise into the dimension-major tile layout.
//                HBM-bound: reads 2*N*D*2 bytes, writes the block.
#include "moqae_dev.hpp"
#include "moqae_kernels.hpp"

namespace moqae {

constexpr int kPlanThreads = 1024;

constexpr int kPlanRun = 8;                          // entries per thread and pass
constexpr int kPlanPass = kPlanThreads * kPlanRun;

// Sum over the workgroup (every thread gets it) and exclusive prefix of x over the threads.
__device__ __forceinline__ unsigned long long plan_block_scan(unsigned long long x, unsigned long long *wsum,
                                                              unsigned long long &total) {
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned long long incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
    __syncthreads();                                  // wsum free
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    unsigned long long before = 0; total = 0;
#pragma unroll
    for (int wv = 0; wv < kPlanThreads / 64; wv++) { const unsigned long long v = wsum[wv]; if (wv < wave) before += v; total += v; }
    return before + incl - x;
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(PackArgs a) {
    __shared__ uint8_t ebuf[kPlanPass];               // a pass's expert indices, in (b, h, c) order
    __shared__ uint32_t obuf[kPlanPass];              // their block offsets relative to the pass, in units of 256 bytes
    __shared__ unsigned long long wsum[kPlanThreads / 64];
    __shared__ int bad;
    const int tid = (int)threadIdx.x;
    if (*a.status != 0) return;                       // sticky error: the call is a no-op
    if (tid == 0) bad = 0;
    __syncthreads();

    const int64_t total = (int64_t)a.BH * a.n_chunks;
    uint32_t size_of[8];                              // rounded block size per expert, in units of 256 bytes
#pragma unroll
    for (int e = 0; e < 8; e++) size_of[e] = (uint32_t)((block_bytes(a.N, a.G, a.bits_of[e]) + 255u) >> 8);
    auto size_at = [&](int e) {
        uint32_t v = 0;
#pragma unroll
        for (int k = 0; k < 8; k++) v = (e == k) ? size_of[k] : v;
        return v;
    };
    const unsigned long long start = (*a.arena_used + 255u) & ~255ull;
    // Entry j of the pass that begins at p0 is (row u, chunk cc) with u*n_chunks + cc = p0 + j; thread t
    // handles entries t, t + 1024, ... (coalesced), stepping (u, cc) without a division.
    const int step_u = kPlanThreads / a.n_chunks, step_c = kPlanThreads % a.n_chunks;

    // Sweep 1: the total size (capacity and expert check) -- nothing is written when the call fails.
    unsigned long long mine = 0, all = 0;
    {
        int64_t u = tid / a.n_chunks; int cc = tid - (int)u * a.n_chunks;
        for (int64_t i = tid; i < total; i += (int64_t)kPlanThreads * 16) {
            int e[16];
#pragma unroll
            for (int k = 0; k < 16; k++) {
                e[k] = (i + (int64_t)k * kPlanThreads < total) ? a.expert[u * a.expert_stride + a.chunk_begin + cc] : 0;
                u += step_u; cc += step_c;
                if (cc >= a.n_chunks) { cc -= a.n_chunks; u++; }
            }
#pragma unroll
            for (int k = 0; k < 16; k++)
                if (i + (int64_t)k * kPlanThreads < total) { if (e[k] >= a.M) bad = 1; else mine += size_at(e[k]); }
        }
    }
    plan_block_scan(mine, wsum, all);
    if (bad) { if (tid == 0) *a.status = -1; return; }
    if (start + (all << 8) > a.capacity) { if (tid == 0) *a.status = -3; return; }

    // Sweep 2: offsets, a pass of kPlanPass entries at a time: staged into LDS with coalesced loads,
    // thread t scans the run of kPlanRun entries from t*kPlanRun, offsets go back through LDS so
    // that the stores are coalesced too.
    unsigned long long carry = start;
    for (int64_t p0 = 0; p0 < total; p0 += kPlanPass) {
        const int n_pass = (int)min((int64_t)kPlanPass, total - p0);
        int64_t u = (p0 + tid) / a.n_chunks; int cc = (int)((p0 + tid) - u * a.n_chunks);
        int64_t at[kPlanRun];
#pragma unroll
        for (int k = 0; k < kPlanRun; k++) {
            const int j = k * kPlanThreads + tid;
            at[k] = u * a.off_stride + a.chunk_begin + cc;
            if (j < n_pass) ebuf[j] = a.expert[u * a.expert_stride + a.chunk_begin + cc];
            u += step_u; cc += step_c;
            if (cc >= a.n_chunks) { cc -= a.n_chunks; u++; }
        }
        __syncthreads();
        const int j0 = min(n_pass, tid * kPlanRun), j1 = min(n_pass, j0 + kPlanRun);
        uint32_t sz[kPlanRun], local = 0;
#pragma unroll
        for (int k = 0; k < kPlanRun; k++) { sz[k] = j0 + k < j1 ? size_at(ebuf[j0 + k]) : 0u; local += sz[k]; }
        unsigned long long pass_total;
        uint32_t pos = (uint32_t)plan_block_scan(local, wsum, pass_total);
#pragma unroll
        for (int k = 0; k < kPlanRun; k++) { if (j0 + k < j1) obuf[j0 + k] = pos; pos += sz[k]; }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kPlanRun; k++) {
            const int j = k * kPlanThreads + tid;
            if (j < n_pass) a.chunk_off[at[k]] = carry + ((unsigned long long)obuf[j] << 8);
        }
        carry += pass_total << 8;
        __syncthreads();                              // ebuf, obuf free
    }
}

// The same plan with one workgroup per (sequence, KV head) row, for tables of at most kPlanRowsMax rows
// whose rows can be read 16 bytes at a time.  Every workgroup reads the whole expert table (it is
// small and stays in L2), so that each knows the sizes of all rows -- the base of its own row and
// the total for the capacity check -- without any exchange between workgroups; it then writes the
// offsets of its own row.
constexpr int kPlanRowsMax = 1024;
__global__ __launch_bounds__(kPlanThreads) void plan_rows_kernel(PackArgs a) {
    __shared__ uint32_t rowtot[kPlanRowsMax];         // block bytes of every row, in units of 256 bytes
    __shared__ unsigned long long wsum[kPlanThreads / 64];
    __shared__ int bad, status_in;
    const int tid = (int)threadIdx.x, u_own = (int)blockIdx.x;
    // One read of the status word per workgroup: workgroup 0 may set it while a workgroup that starts later is
    // reading it, and all wavefronts of a workgroup must take the same way out.  (A workgroup that still sees 0
    // reaches the same verdict as workgroup 0 by itself and writes nothing either.)
    if (tid == 0) { status_in = *a.status; bad = 0; }
    for (int i = tid; i < a.BH; i += kPlanThreads) rowtot[i] = 0;
    __syncthreads();
    if (status_in != 0) return;                       // sticky error: the call is a no-op

    uint32_t size_of[8];
    unsigned long long lut = 0;                       // size_of[e] in 16-bit field e (a block is < 2^16 * 256 bytes)
#pragma unroll
    for (int e = 0; e < 8; e++) {
        size_of[e] = (uint32_t)((block_bytes(a.N, a.G, a.bits_of[e]) + 255u) >> 8);
        if (e < 4) lut |= (unsigned long long)size_of[e] << (16 * e);
    }
    unsigned long long lut_hi = 0;
#pragma unroll
    for (int e = 4; e < 8; e++) lut_hi |= (unsigned long long)size_of[e] << (16 * (e - 4));
    auto size_at = [&](uint32_t e) { return (uint32_t)(((e & 4u) ? lut_hi : lut) >> (16u * (e & 3u))) & 0xffffu; };
    const unsigned long long start = (*a.arena_used + 255u) & ~255ull;

    // (1) sizes of all rows: 16-byte pieces of the table, all requested before any is used
    const int C = a.n_chunks, C16 = C & ~15, ppr = C16 / 16;             // whole pieces per row
    const int n_pieces = a.BH * ppr;
    for (int p0 = 0; p0 < n_pieces; p0 += kPlanThreads * 8) {
        uint4 v[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const int p = min(p0 + k * kPlanThreads + tid, n_pieces - 1);
            const int row = p / ppr, c = (p - row * ppr) * 16;
            v[k] = *reinterpret_cast<const uint4 *>(a.expert + (int64_t)row * a.expert_stride + a.chunk_begin + c);
        }
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const int p = p0 + k * kPlanThreads + tid;
            if (p < n_pieces) {
                const uint32_t wv[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
                uint32_t sum = 0;
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const uint32_t e = (wv[i >> 2] >> (8 * (i & 3))) & 0xffu;
                    if (e >= (uint32_t)a.M) bad = 1;
                    sum += size_at(e);
                }
                atomicAdd(&rowtot[p / ppr], sum);
            }
        }
    }
    for (int i = tid; i < a.BH * (C - C16); i += kPlanThreads) {         // the last < 16 chunks of every row
        const int row = i / (C - C16), c = C16 + i % (C - C16);
        const uint32_t e = a.expert[(int64_t)row * a.expert_stride + a.chunk_begin + c];
        if (e >= (uint32_t)a.M) bad = 1;
        atomicAdd(&rowtot[row], size_at(e));
    }
    __syncthreads();

    // (2) base of every row and the total; the verdict is the same in every workgroup
    unsigned long long all = 0;
    const unsigned long long before = plan_block_scan(tid < a.BH ? (unsigned long long)rowtot[tid] : 0ull, wsum, all);
    __shared__ unsigned long long own_base;
    if (tid == u_own) own_base = before;
    if (bad) { if (tid == 0 && u_own == 0) *a.status = -1; return; }
    if (start + (all << 8) > a.capacity) { if (tid == 0 && u_own == 0) *a.status = -3; return; }
    __syncthreads();

    // (3) the offsets of this workgroup's row
    unsigned long long carry = start + (own_base << 8);
    for (int c0 = 0; c0 < C; c0 += kPlanThreads) {
        const int c = c0 + tid;
        const uint32_t sz = c < C ? size_at(a.expert[(int64_t)u_own * a.expert_stride + a.chunk_begin + c]) : 0u;
        unsigned long long pass_total;
        const unsigned long long pos = plan_block_scan(sz, wsum, pass_total);
        if (c < C) a.chunk_off[(int64_t)u_own * a.off_stride + a.chunk_begin + c] = carry + (pos << 8);
        carry += pass_total << 8;
    }
}

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
template <int G, int BITS>
__device__ __forceinline__ void pack_item(const uint4 *__restrict__ p, bool isV, uint32_t *__restrict__ meta_dst,
                                          uint32_t *__restrict__ k_dst, uint32_t *__restrict__ v_lds) {
    constexpr int NW = G / 2;                        // input words (fp16 pairs) of the item
    static_assert(NW >= 16, "G >= 32");
    uint32_t w[NW];
#pragma unroll
    for (int j = 0; j < G / 8; j++) {                // the whole item is requested at once: its 128-byte line arrives once
        // (ordinary loads: the lane's eight loads share the line through the cache; streaming loads here fetch it eight times)
        const uint4 t = p[j];
        w[4 * j] = t.x; w[4 * j + 1] = t.y; w[4 * j + 2] = t.z; w[4 * j + 3] = t.w;
    }
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
    nt_store(meta_dst, s16 | (float_to_half_bits(mn) << 16));
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
            for (int k = 0; k < WPL; k += 4)
                nt_store(reinterpret_cast<uint4 *>(k_dst + k), uint4{out[k], out[k + 1], out[k + 2], out[k + 3]});
        } else {
            static_assert(WPL == 2, "G = 32 at 2 bits");
            nt_store(reinterpret_cast<uint2 *>(k_dst), uint2{out[0], out[1]});
        }
    }
}

template <int G>
__global__ __launch_bounds__(kPackThreads) void pack_kernel(PackArgs a) {
    extern __shared__ uint8_t vcodes[];               // [N][kVRow] code bytes (V only); odd dword stride: rows fall on different banks
    if (*a.status != 0) return;

    const int isV = (int)blockIdx.x;                  // K and V of a chunk side by side in launch order: the lighter K
    const int c = a.chunk_begin + (int)blockIdx.y;    // workgroups and the V workgroups (LDS phase) share the CUs at all times
    const int u = (int)blockIdx.z;
    const int tid = (int)threadIdx.x;
    const int N = a.N;
    const int bits = a.bits_of[a.expert[(int64_t)u * a.expert_stride + c]];
    uint8_t *blk = a.arena + a.chunk_off[(int64_t)u * a.off_stride + c];
    const int b = u / a.Hkv, h = u % a.Hkv;
    const uint16_t *src = (isV ? a.V : a.K) + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h
                        + (int64_t)c * N * a.stride_s;

    if (bits == 16) {                                 // FP16 expert: rows copied verbatim
        const int lane16 = tid & 15, rsub = tid >> 4;
        uint4 *dst = reinterpret_cast<uint4 *>(blk + (isV ? (size_t)N * kD * 2 : 0));
        for (int row = rsub; row < N; row += kPackThreads / 16)
            nt_store(&dst[row * 16 + lane16], nt_load(reinterpret_cast<const uint4 *>(src + (int64_t)row * a.stride_s + lane16 * 8)));
        return;
    }

    constexpr int NG = kD / G;                        // groups per row
    const size_t code_bytes = (size_t)N * kD * bits / 8, meta_bytes = (size_t)N * NG * 4;
    uint8_t *area = blk + (isV ? code_bytes + meta_bytes : 0);
    uint32_t *codes_w = reinterpret_cast<uint32_t *>(area);
    uint32_t *meta_w = reinterpret_cast<uint32_t *>(area + code_bytes);

    // item = (token row, group): consecutive lanes take consecutive 2G-byte pieces of the chunk
    for (int item = tid; item < N * NG; item += kPackThreads) {
        const int row = item / NG, g = item % NG;
        const uint4 *p = reinterpret_cast<const uint4 *>(src + (int64_t)row * a.stride_s + g * G);
        uint32_t *vl = reinterpret_cast<uint32_t *>(vcodes + row * kVRow + g * G);
        if (bits == 2)      pack_item<G, 2>(p, isV, &meta_w[item], codes_w + item * (G / 16), vl);
        else if (bits == 4) pack_item<G, 4>(p, isV, &meta_w[item], codes_w + item * (G / 8), vl);
        else                pack_item<G, 8>(p, isV, &meta_w[item], codes_w + item * (G / 4), vl);
    }
    if (!isV) return;

    __syncthreads();
    // V: dimension-major tiles of 16*QD slots x 4 words.  A slot holds TQ = max(TW, 8) consecutive tokens
    // (TW = 32/bits per word, WD = TQ/TW words) of CPK = 4/WD dimensions that lie 16 apart; a token block is
    // TB = min(4*TQ, N) tokens = QD slices (QD = 4, i.e. 1-KiB tiles, except for 32-token chunks at 2 bits: QD = 2);
    // slot 16*qd + j of tile cg of a block: dims 16*(cg*CPK + n/WD) + j, token slice qd.
    const int TW = 32 / bits, TQ = TW > 8 ? TW : 8, WD = TQ / TW, CPK = 4 / WD, NCG = kD / (16 * CPK);
    const int TB = min(4 * TQ, N), QD = TB / TQ;
    const int n_groups = N * kD * bits / 128;         // a thread builds the words of four adjacent dims at a time
    for (int g = tid; g < n_groups; g += kPackThreads) {
        const int n = g & 3, jq = (g >> 2) & 3, qd = (g >> 4) & (QD - 1), tile = g / (16 * QD);
        const int cg = tile % NCG, block = tile / NCG;
        const int d0 = 16 * (cg * CPK + n / WD) + 4 * jq, t0 = block * TB + qd * TQ + (n % WD) * TW;
        uint32_t w0 = 0, w1 = 0, w2 = 0, w3 = 0;
        for (int e = 0; e < TW; e++) {
            const uint32_t v4 = *reinterpret_cast<const uint32_t *>(vcodes + (t0 + e) * kVRow + d0);   // codes of dims d0..d0+3
            const int sh = code_shift(e, bits);
            w0 |= (v4 & 0xffu) << sh; w1 |= ((v4 >> 8) & 0xffu) << sh; w2 |= ((v4 >> 16) & 0xffu) << sh; w3 |= (v4 >> 24) << sh;
        }
        // thread n = 0..3 of a quad holds word n of the slots 16*qd + 4*jq + k, k = 0..3: a 4 x 4 transpose inside
        // the quad leaves every thread with one whole slot, stored with one 16-byte store
        uint32_t wk[4] = {w0, w1, w2, w3};
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

// The new end of the arena = the end of the last block in (b, h, c) order.  A kernel of its own, after
// the plan: the workgroups of the plan read the counter at different times, so none of them may move
// it, and the few registers this takes would cost the pack kernel occupancy.
__global__ void arena_end_kernel(PackArgs a) {
    if (*a.status != 0) return;
    const int64_t lu = a.BH - 1, lc = a.chunk_begin + a.n_chunks - 1;
    const unsigned long long sz = (block_bytes(a.N, a.G, a.bits_of[a.expert[lu * a.expert_stride + lc]]) + 255u) & ~255ull;
    *a.arena_used = a.chunk_off[lu * a.off_stride + lc] + sz;
}

// The new token's K and V rows (fp16 [B*Hkv, D]) into row n_tail of the FP16 residual buffers ([B*Hkv, N, D]): one
// kernel for both, one 16-byte piece per thread.
__global__ __launch_bounds__(32) void append_tail_kernel(const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
                                                         uint4 *__restrict__ K_tail, uint4 *__restrict__ V_tail, int N, int n_tail) {
    const int u = (int)blockIdx.x, t = (int)threadIdx.x;   // 16 pieces of K, 16 of V
    const size_t dst = ((size_t)u * N + n_tail) * (kD / 8) + (t & 15);
    if (t < 16) K_tail[dst] = k_new[(size_t)u * (kD / 8) + t];
    else        V_tail[dst] = v_new[(size_t)u * (kD / 8) + (t & 15)];
}
hipError_t launch_append_tail(const void *k_new, const void *v_new, void *K_tail, void *V_tail, int BH, int N, int n_tail,
                              hipStream_t s) {
    hipLaunchKernelGGL(append_tail_kernel, dim3((unsigned)BH), dim3(32), 0, s, static_cast<const uint4 *>(k_new),
                       static_cast<const uint4 *>(v_new), static_cast<uint4 *>(K_tail), static_cast<uint4 *>(V_tail), N, n_tail);
    return hipGetLastError();
}

hipError_t launch_pack(const PackArgs &a, hipStream_t s) {
    if (a.n_chunks <= 0 || a.BH <= 0) return hipSuccess;
    const bool rows_ok = a.BH <= kPlanRowsMax &&
                         ((reinterpret_cast<uintptr_t>(a.expert + a.chunk_begin) | (uintptr_t)a.expert_stride) & 15u) == 0;
    if (rows_ok) hipLaunchKernelGGL(plan_rows_kernel, dim3((unsigned)a.BH), dim3(kPlanThreads), 0, s, a);
    else         hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid(2u, (unsigned)a.n_chunks, (unsigned)a.BH);
    const size_t lds = (size_t)a.N * kVRow;
    if (a.G == 32) hipLaunchKernelGGL(pack_kernel<32>, grid, dim3(kPackThreads), lds, s, a);
    else           hipLaunchKernelGGL(pack_kernel<64>, grid, dim3(kPackThreads), lds, s, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(arena_end_kernel, dim3(1), dim3(1), 0, s, a);
    return hipGetLastError();
}

}  // namespace moqae
