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
#include "pack_dev.hpp"

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

template <int G, bool KPC>
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

    pack_side<G, KPC>(src, a.stride_s, N, bits, isV, blk, vcodes, tid, kPackThreads);
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
    if (a.kpc) {
        if (a.G == 32) hipLaunchKernelGGL((pack_kernel<32, true>), grid, dim3(kPackThreads), lds, s, a);
        else           hipLaunchKernelGGL((pack_kernel<64, true>), grid, dim3(kPackThreads), lds, s, a);
    } else {
        if (a.G == 32) hipLaunchKernelGGL((pack_kernel<32, false>), grid, dim3(kPackThreads), lds, s, a);
        else           hipLaunchKernelGGL((pack_kernel<64, false>), grid, dim3(kPackThreads), lds, s, a);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(arena_end_kernel, dim3(1), dim3(1), 0, s, a);
    return hipGetLastError();
}

}  // namespace moqae
