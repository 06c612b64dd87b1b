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
    int bits_of[8];
};
hipError_t launch_pack(const PackArgs &a, hipStream_t s);
hipError_t launch_append_tail(const void *k_new, const void *v_new, void *K_tail, void *V_tail, int BH, int N, int n_tail,
                              hipStream_t s);

struct AttnArgs {
    const uint16_t *q; const uint8_t *arena; const uint64_t *chunk_off; const uint8_t *expert;
    int64_t desc_stride;
    const uint16_t *K_tail, *V_tail;
    const int32_t *seq_chunks, *seq_tail;   // ragged batch: chunks / residual rows per sequence (device), else null
    float *part; float *out;
    unsigned int *counters;     // ticket counters, one per (row, row segment), attn_counter_bytes() in all
    float scale_log2;           // softmax_scale * log2(e)
    int n_chunks, n_tail, n_wg, max_partials, N, G, Hkv, rep, BH;
    int planned;                // the workspace holds a plan: no prep kernel, the merge kernel zeroes the counters again
    int bits_of[8];
};
hipError_t launch_attn_plan(const AttnArgs &a, hipStream_t s);
hipError_t launch_attn(const AttnArgs &a, hipStream_t s, hipEvent_t ev_begin = nullptr, hipEvent_t ev_end = nullptr);
int attn_waves_per_wg(int rep);
int attn_max_partials(int n_wg, int BH);        // partial slots per row
size_t attn_counter_bytes(int BH, int n_chunks, int N); // bytes of the ticket counters at the start of the workspace


}  // namespace moqae
