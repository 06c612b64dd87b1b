// moqae_route_pack_paged: router (Eq. (1)-(2), Sec. 3.2; routing freezing, Sec. 3.4), page allocation and
// quantise-and-pack of a chunk in ONE kernel, on a store of per-expert pools of fixed pages.
//
// The ordered arena of moqae_quantize_pack puts a chunk's block where the blocks of all earlier chunks end,
// so packing has to wait for every routing decision.  With one pool of equal pages per expert a chunk's place
// is one atomic step on its pool's free ring, and the workgroup that has just routed the chunk quantises it at
// once, so K comes from memory once.
//
//   route_pack_kernel  one workgroup per (sequence, KV head, chunk), one thread per token.  Keys per token: the thread
//                      gets its whole key row (a wavefront reads its 64 rows in whole lines and hands every lane its
//                      own through LDS: rows_request, rows_transpose), routes it (route_row, the operations of
//                      route_kernel in the same order), the votes are added up in LDS, one thread takes a page of the
//                      routed expert's pool, then every thread quantises the row it still holds in registers and
//                      after it its value row (pack_row, the arithmetic of pack_kernel).  A thread's codes are pieces
//                      of lines, so the K codes and the V codes both go through staging rows in LDS and leave in
//                      whole lines (k_flush, v_gather).  No key row is kept in LDS: 18 KiB per 128-token workgroup,
//                      eight workgroups per compute unit.
//                      Keys per channel (a group runs over G tokens, so a thread cannot quantise its own row): the
//                      routing wavefronts leave the key rows in LDS (route_tokens) and pack_side takes them from there.
//   pool_*_kernel      the free rings.  Device-wide atomic steps on ONE address run at about nine per microsecond on
//                      this eight-die chip (40 960 chunks on four pool counters took 3.5 ms, 0.8 ms without them), so
//                      every pool's free pages are spread over kPoolShards rings: a chunk starts at a ring chosen by
//                      its indices and walks on while rings are empty; a page goes back to the ring it came from.
#include "moqae_dev.hpp"
#include "moqae_kernels.hpp"
#include "pack_dev.hpp"
#include "route_dev.hpp"

namespace moqae {

template <int M, int G, bool KPC>
__global__ __launch_bounds__(kPackThreads) void route_pack_kernel(PagedArgs a) {
    extern __shared__ uint4 dyn_lds[];                // keys per channel: the chunk's key rows as the router read them (N * kStageRow
    uint8_t *vcodes = reinterpret_cast<uint8_t *>(dyn_lds);   // pieces); then the staging rows of the codes (K: k_stage_row, V: kVRow bytes per token)
    __shared__ float w3f[72];
    __shared__ int votes_s[8];
    __shared__ unsigned long long page_off;
    __shared__ int expert_s, status_in;

    const int c = a.chunk_begin + (int)blockIdx.x, u = (int)blockIdx.y;
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6, NT = (int)blockDim.x;
    const int N = a.N;
    const int64_t eidx = (int64_t)u * a.expert_stride + c;
    const int b = u / a.Hkv, h = u % a.Hkv;
    const int64_t base = (int64_t)b * a.stride_b + (int64_t)h * a.stride_h + (int64_t)c * N * a.stride_s;

    // ---- (1) the decision: given, frozen, or routed here
    const bool routed = a.W1 != nullptr && c >= a.freeze_chunks;
    if (tid < 8) votes_s[tid] = 0;
    if (tid == 0) status_in = (int)a.state[0];        // the status word when the call began (paged_begin_kernel): other
                                                      // workgroups of this call may be setting the word itself right now
    if (routed) {
        if (tid < M * M) w3f[tid] = half_bits_to_float(a.W3[tid]);
        if (a.bias && tid < M) w3f[64 + tid] = a.bias[tid];
    }
    __syncthreads();
    if (status_in != 0) return;                       // sticky error: the call is a no-op
    // Keys per token: thread t owns token t.  Its whole key row stays in registers from the router to the quantiser.
    uint4 x[16], xv[16];
    const bool own = tid < N;
    if constexpr (!KPC) {
        rows_request(a.K + base, a.stride_s, N, wave, lane, xv);
        rows_transpose(xv, vcodes, wave, lane, x);
        if (routed) {
            const int top = route_row<M>(x, reinterpret_cast<const uint32_t *>(a.W1), reinterpret_cast<const uint32_t *>(a.W2), w3f,
                                         a.bias != nullptr);
#pragma unroll
            for (int k = 0; k < M; k++) {
                const int n = __popcll(__ballot(own && top == k));
                if (lane == k) atomicAdd(&votes_s[k], n);
            }
        }
    } else if (routed && wave * 64 < N) {
        int cnt[M];
        route_tokens<M, true>(a.K + base + (int64_t)wave * 64 * a.stride_s, min(64, N - wave * 64), a.stride_s,
                              reinterpret_cast<const uint32_t *>(a.W1), reinterpret_cast<const uint32_t *>(a.W2), w3f,
                              a.bias != nullptr, lane, cnt, dyn_lds + wave * 64 * kStageRow);
#pragma unroll
        for (int k = 0; k < M; k++) if (lane == k) atomicAdd(&votes_s[k], cnt[k]);
    }
    __syncthreads();
    // ---- (2) one thread settles the expert and takes a page
    if (tid == 0) {
        int e;
        if (routed) {
            e = 0;
            for (int k = 1; k < M; k++) if (votes_s[k] > votes_s[e]) e = k;   // strict: the first maximum wins
            a.expert[eidx] = (uint8_t)e;
        } else if (a.W1 != nullptr) {                 // frozen chunk: the first 16-bit expert, never routed
            e = a.e16;
            a.expert[eidx] = (uint8_t)e;
        } else {
            e = a.expert[eidx];                       // a routing-sharing leader's decision
        }
        unsigned long long off = ~0ull;
        if (e >= M) {
            atomicCAS(a.status, 0, -1);
        } else {
            // tails do not move during this call; a head that ran past its tail (the ring was empty when several
            // workgroups tried) is pulled back by the next call's first kernel
            uint32_t *heads = a.state + 16 + e * 2 * kPoolShards, *tails = heads + kPoolShards;
            const uint32_t s0 = (uint32_t)(u * 131 + c * 7);
            bool got = false;
            for (uint32_t k = 0; k < (uint32_t)kPoolShards && !got; k++) {
                const uint32_t sh = (s0 + k) % kPoolShards, tail = tails[sh];
                if ((int32_t)(tail - __atomic_load_n(&heads[sh], __ATOMIC_RELAXED)) <= 0) continue;   // looks empty: no atomic step
                const uint32_t hv = atomicAdd(&heads[sh], 1u);
                if ((int32_t)(tail - hv) > 0) {
                    const uint32_t page = a.state[a.ring_start[e] + sh * a.ring_cap[e] + hv % a.ring_cap[e]];
                    off = a.pool_base[e] + (unsigned long long)page * a.page_bytes[e];
                    got = true;
                }
            }
            if (!got) atomicCAS(a.status, 0, -3);
        }
        a.chunk_off[(int64_t)u * a.off_stride + c] = off;
        page_off = off; expert_s = e;
    }
    if (a.votes && a.W1 != nullptr && tid < M) a.votes[eidx * M + tid] = routed ? votes_s[tid] : 0;
    __syncthreads();
    if (page_off == ~0ull) return;
    // ---- (3) quantise and pack K, then V, into the page
    const int bits = a.bits_of[expert_s];
    uint8_t *blk = a.arena + page_off;
    if constexpr (!KPC) {
        if (own) pack_row<G>(x, tid, N, bits, 0, blk, vcodes);
        rows_request(a.V + base, a.stride_s, N, wave, lane, xv);   // in flight while the K codes leave
        if (bits != 16) {
            __syncthreads();
            k_flush(N, bits, blk, vcodes, tid, NT);
            __syncthreads();                          // the K staging rows are consumed: the buffers of the transposition take their place
        }
        rows_transpose(xv, vcodes, wave, lane, x);
        if (bits != 16) __syncthreads();              // every wavefront has its rows: the V staging rows take the buffers' place
        if (own) pack_row<G>(x, tid, N, bits, 1, blk, vcodes);
        if (bits == 16) return;
        __syncthreads();
        const int room = v_token_room(N, bits);
        v_gather(N, bits, room, reinterpret_cast<uint32_t *>(blk + (size_t)N * kD * bits / 8 + (size_t)N * (kD / G) * 4), vcodes, tid, NT);
    } else {
        if (routed) {                                 // the keys are in LDS: K comes from memory once
            pack_side<G, KPC>(reinterpret_cast<const uint16_t *>(dyn_lds), kStageRow * 8, N, bits, 0, blk, vcodes, tid, NT);
            __syncthreads();                          // the key rows are consumed: the V staging rows take their place
        } else {
            pack_side<G, KPC>(a.K + base, a.stride_s, N, bits, 0, blk, vcodes, tid, NT);
        }
        pack_side<G, KPC>(a.V + base, a.stride_s, N, bits, 1, blk, vcodes, tid, NT);
    }
}

// Before every call: the status word is latched for the call's workgroups, and heads that ran past their tails on
// empty rings in an earlier call come back to them.
__global__ void paged_begin_kernel(PagedArgs a) {
    const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);   // 8 * kPoolShards threads
    if (i == 0) a.state[0] = (uint32_t)*a.status;
    const int j = i / kPoolShards, sh = i % kPoolShards;
    uint32_t *heads = a.state + 16 + j * 2 * kPoolShards;
    if (j < a.M && (int32_t)(heads[kPoolShards + sh] - heads[sh]) < 0) heads[sh] = heads[kPoolShards + sh];
}
__global__ void pool_clamp_kernel(PagedArgs a) {
    const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x), j = i / kPoolShards, sh = i % kPoolShards;
    uint32_t *heads = a.state + 16 + j * 2 * kPoolShards;
    if (j < a.M && (int32_t)(heads[kPoolShards + sh] - heads[sh]) < 0) heads[sh] = heads[kPoolShards + sh];
}

// Every page free: page p in ring p % kPoolShards at position p / kPoolShards.
__global__ void pool_init_kernel(PagedArgs a) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 16) a.state[i] = 0u;
    if (i < 8u * kPoolShards) {
        const uint32_t j = i / kPoolShards, sh = i % kPoolShards;
        uint32_t *heads = a.state + 16 + j * 2 * kPoolShards;
        heads[sh] = 0u;
        heads[kPoolShards + sh] = (j < (uint32_t)a.M && sh < a.n_pages[j]) ? (a.n_pages[j] - sh + kPoolShards - 1) / kPoolShards : 0u;
    }
    for (int j = 0; j < a.M; j++)
        if (i < a.n_pages[j]) a.state[a.ring_start[j] + (i % kPoolShards) * a.ring_cap[j] + i / kPoolShards] = i;
}

// One thread per (row, chunk) of the range: its page goes back to the ring it came from.
__global__ void pool_release_kernel(PagedArgs a, int row_begin, int n_rows) {
    const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (i >= n_rows * a.n_chunks) return;
    const int u = row_begin + i / a.n_chunks, c = a.chunk_begin + i % a.n_chunks;
    const unsigned long long off = a.chunk_off[(int64_t)u * a.off_stride + c];
    const int e = a.expert[(int64_t)u * a.expert_stride + c];
    if (off == ~0ull || e >= a.M) return;
    const uint32_t page = (uint32_t)((off - a.pool_base[e]) / a.page_bytes[e]), sh = page % kPoolShards;
    uint32_t *tails = a.state + 16 + e * 2 * kPoolShards + kPoolShards;
    const uint32_t t = atomicAdd(&tails[sh], 1u);
    a.state[a.ring_start[e] + sh * a.ring_cap[e] + t % a.ring_cap[e]] = page;
    a.chunk_off[(int64_t)u * a.off_stride + c] = ~0ull;
}

// Free pages per pool -> counts[0..7].
__global__ void pool_free_pages_kernel(PagedArgs a, uint32_t *counts) {
    const int j = (int)blockIdx.x, lane = (int)threadIdx.x;        // one wavefront per pool
    const uint32_t *heads = a.state + 16 + j * 2 * kPoolShards;
    int n = 0;
    if (j < a.M) for (int sh = lane; sh < kPoolShards; sh += 64) n += max((int32_t)(heads[kPoolShards + sh] - heads[sh]), 0);
    for (int o = 32; o >= 1; o >>= 1) n += __shfl_xor(n, o);
    if (lane == 0) counts[j] = (uint32_t)n;
}

template <int M>
static hipError_t launch_rp(const PagedArgs &a, dim3 grid, size_t lds, hipStream_t s) {
    // as many wavefronts as the chunk has passes of 64 tokens: all of them route, then all of them pack
    const dim3 block((unsigned)(a.N <= 64 ? 64 : (a.N >= 256 ? 256 : (a.N + 63) / 64 * 64)));
    if (lds > 65536) {                                // 256-token chunks: 68 KiB of key rows; above the default limit of dynamic LDS
        static bool raised[2][2] = {{false, false}, {false, false}};
        bool &r = raised[a.G == 32][a.kpc != 0];
        if (!r) {
            hipError_t e = hipSuccess;
            if (a.kpc) e = a.G == 32 ? hipFuncSetAttribute((const void *)route_pack_kernel<M, 32, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                                     : hipFuncSetAttribute((const void *)route_pack_kernel<M, 64, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            else       e = a.G == 32 ? hipFuncSetAttribute((const void *)route_pack_kernel<M, 32, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                                     : hipFuncSetAttribute((const void *)route_pack_kernel<M, 64, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            r = true;
        }
    }
    if (a.kpc) {
        if (a.G == 32) hipLaunchKernelGGL((route_pack_kernel<M, 32, true>), grid, block, lds, s, a);
        else           hipLaunchKernelGGL((route_pack_kernel<M, 64, true>), grid, block, lds, s, a);
    } else {
        if (a.G == 32) hipLaunchKernelGGL((route_pack_kernel<M, 32, false>), grid, block, lds, s, a);
        else           hipLaunchKernelGGL((route_pack_kernel<M, 64, false>), grid, block, lds, s, a);
    }
    return hipGetLastError();
}

hipError_t launch_route_pack_paged(const PagedArgs &a, hipStream_t s) {
    if (a.n_chunks <= 0 || a.BH <= 0) return hipSuccess;
    hipLaunchKernelGGL(paged_begin_kernel, dim3(8 * kPoolShards / 256), dim3(256), 0, s, a);
    hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return e0;
    dim3 grid((unsigned)a.n_chunks, (unsigned)a.BH);
    // keys per token: a transposition buffer per wavefront, then the staging rows of the K codes, then of the V codes;
    // keys per channel: the key rows as the router read them, then the V rows
    const int nt = a.N <= 64 ? 64 : (a.N >= 256 ? 256 : (a.N + 63) / 64 * 64);   // threads of a workgroup (launch_rp)
    const size_t lds = a.kpc ? (size_t)a.N * (kStageRow * 16 > kVRow ? kStageRow * 16 : kVRow)
                             : (size_t)nt * (k_stage_row(8) > kTRow ? k_stage_row(8) : kTRow);
    switch (a.M) {
        case 1: return launch_rp<1>(a, grid, lds, s);
        case 2: return launch_rp<2>(a, grid, lds, s);
        case 3: return launch_rp<3>(a, grid, lds, s);
        case 4: return launch_rp<4>(a, grid, lds, s);
        case 5: return launch_rp<5>(a, grid, lds, s);
        case 6: return launch_rp<6>(a, grid, lds, s);
        case 7: return launch_rp<7>(a, grid, lds, s);
        case 8: return launch_rp<8>(a, grid, lds, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_pool_init(const PagedArgs &a, hipStream_t s) {
    uint32_t most = 8 * kPoolShards;
    for (int j = 0; j < a.M; j++) most = a.n_pages[j] > most ? a.n_pages[j] : most;
    hipLaunchKernelGGL(pool_init_kernel, dim3((most + 255u) / 256u), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_pool_release(const PagedArgs &a, int row_begin, int n_rows, hipStream_t s) {
    const long long n = (long long)n_rows * a.n_chunks;
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(pool_clamp_kernel, dim3(8 * kPoolShards / 256), dim3(256), 0, s, a);   // heads left past their tails by a call that found rings empty
    hipLaunchKernelGGL(pool_release_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a, row_begin, n_rows);
    return hipGetLastError();
}

hipError_t launch_pool_free_pages(const PagedArgs &a, uint32_t *counts, hipStream_t s) {
    hipLaunchKernelGGL(pool_free_pages_kernel, dim3(8), dim3(64), 0, s, a, counts);
    return hipGetLastError();
}

}  // namespace moqae
