// Host-visible launch interface of the three kernels (internal to libmoqae).
#pragma once
#include <cstddef>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moqae {

struct RouteArgs {
    const uint16_t *K; int64_t stride_b, stride_h, stride_s;
    const uint16_t *W1, *W2, *W3; const float *bias;
    uint8_t *expert; int64_t expert_stride; int32_t *votes;
    int chunk_begin, N, Hkv, freeze_chunks, e16;
};
hipError_t launch_route(const RouteArgs &a, int M, int n_chunks, int BH, hipStream_t s);

struct PackArgs {
    const uint16_t *K, *V; int64_t stride_b, stride_h, stride_s;
    const uint8_t *expert; int64_t expert_stride;
    uint8_t *arena; uint64_t capacity; uint64_t *arena_used;
    uint64_t *chunk_off; int64_t off_stride; int32_t *status;
    int chunk_begin, n_chunks, BH, N, G, Hkv, M;
    int kpc;                    // keys quantised per channel (groups of G tokens of one dim)
    int bits_of[8];
};
hipError_t launch_pack(const PackArgs &a, hipStream_t s);
hipError_t launch_append_tail(const void *k_new, const void *v_new, void *K_tail, void *V_tail, int BH, int N, int n_tail,
                              hipStream_t s);

// Paged store: pool j (expert j) = n_pages[j] pages of page_bytes[j] bytes from pool_base[j].  Its free pages sit in
// kPoolShards rings (page p lives in ring p % kPoolShards, which holds ring_cap[j] entries), so that the atomic steps of
// a call spread over many addresses.  State words: [0] the status word as it was when the running call began, [1..15]
// reserved; from word 16 pool j's shard heads then shard tails (2 * kPoolShards words per pool); rings from ring_start[j].
constexpr int kPoolShards = 256;
struct PagedArgs {
    const uint16_t *K, *V; int64_t stride_b, stride_h, stride_s;
    const uint16_t *W1, *W2, *W3; const float *bias;      // W1 == null: `expert` holds the decisions to use
    uint8_t *expert; int64_t expert_stride; int32_t *votes;
    uint8_t *arena; uint32_t *state;
    unsigned long long *chunk_off; int64_t off_stride; int32_t *status;
    int chunk_begin, n_chunks, BH, N, G, Hkv, M, freeze_chunks, e16, kpc;
    int bits_of[8];
    uint32_t n_pages[8], ring_start[8], ring_cap[8], page_bytes[8];
    unsigned long long pool_base[8];
};
hipError_t launch_route_pack_paged(const PagedArgs &a, hipStream_t s);
hipError_t launch_pool_init(const PagedArgs &a, hipStream_t s);
hipError_t launch_pool_release(const PagedArgs &a, int row_begin, int n_rows, hipStream_t s);
hipError_t launch_pool_free_pages(const PagedArgs &a, uint32_t *counts, hipStream_t s);

struct TrainArgs {
    const uint16_t *K; int64_t stride_b, stride_h, stride_s;
    const uint16_t *W1, *W2, *W3; const float *bias; const float *nll;
    float pen_model[8], pen_mem[8]; float lambda, inv_T;
    int token_begin, n_tok, BH, Hkv, M;
    float *loss3, *dW1, *dW2, *dW3, *dbias;
};
hipError_t launch_router_train(const TrainArgs &a, int n_cu, hipStream_t s);

struct AttnArgs {
    const uint16_t *q; const uint8_t *arena; const uint64_t *chunk_off; const uint8_t *expert;
    int64_t desc_stride;
    const uint16_t *K_tail, *V_tail;
    const int32_t *seq_chunks, *seq_tail;   // ragged batch: chunks / residual rows per sequence (device), else null
    float *part; float *out;
    unsigned int *counters;     // ticket counters, one per (row, row segment), attn_counter_bytes() in all
    float scale_log2;           // softmax_scale * log2(e)
    int n_chunks, n_tail, n_wg, max_partials, N, G, Hkv, rep, BH;
    int kpc;                    // keys quantised per channel
    int nq, rep_in;             // queries per sequence (1: decode of one token) and query heads per KV head of one query; rep = nq * rep_in
    int planned;                // the workspace holds a plan: no prep kernel, the merge kernel zeroes the counters again
    int bits_of[8];
};
hipError_t launch_attn_plan(const AttnArgs &a, hipStream_t s);
hipError_t launch_attn(const AttnArgs &a, hipStream_t s, hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr);
int attn_waves_per_wg(int rep);
int attn_max_partials(int n_wg, int BH);        // partial slots per row
size_t attn_counter_bytes(int BH, int n_chunks, int N); // bytes of the ticket counters at the start of the workspace


}  // namespace moqae
