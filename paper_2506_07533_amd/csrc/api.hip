// C-ABI entry points of libmoqae: argument validation on the host, then kernel launches on the
// caller's stream.  No allocation and no synchronisation happen here.
#include "../../include/moqae.h"
#include "../../include/moqae_bench.h"
#include "moqae_dev.hpp"
#include "moqae_kernels.hpp"
#include <mutex>

using namespace moqae;

// Scratch memory of moqae_decode_attn_static: the decode workspace (ticket counters, row costs, softmax partials) of
// callers that cannot allocate.  One copy per GPU the library runs on, held until the process ends.  In host code the
// array's name is only a stand-in for hipGetSymbolAddress; kernels get the address that call returns.
#define MOQAE_STATIC_SCRATCH_BYTES (8u << 20)
static __device__ __align__(256) unsigned char scratch[MOQAE_STATIC_SCRATCH_BYTES];

namespace {

bool bits_ok(int b) { return b == 2 || b == 4 || b == 8 || b == 16; }

bool cfg_ok(const moqae_cfg *c) {
    if (!c) return false;
    if (c->batch < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1) return false;
    if (c->n_q_heads % c->n_kv_heads) return false;
    const int rep = c->n_q_heads / c->n_kv_heads;
    if (rep != 1 && rep != 2 && rep != 4 && rep != 8) return false;
    if ((int64_t)c->batch * c->n_kv_heads > 65535) return false;          // grid.y
    if (c->head_dim != kD) return false;
    if (c->group != 32 && c->group != 64) return false;
    if (c->chunk != 8 && c->chunk != 16 && (c->chunk < 32 || c->chunk > 256 || c->chunk % 32)) return false;
    if (c->n_experts < 1 || c->n_experts > MOQAE_MAX_EXPERTS) return false;
    for (int j = 0; j < c->n_experts; j++) if (!bits_ok(c->expert_bits[j])) return false;
    if (c->freeze_chunks < 0) return false;
    if (c->k_per_channel != 0 && c->k_per_channel != 1) return false;
    if (c->k_per_channel && c->chunk % c->group) return false;            // token groups must tile the chunk
    return true;
}

// The packed layout (pack and decode calls): V token blocks span up to 64 tokens (chunks of 8, 16 and 32 tokens
// are one block with its own tile shape), and the decode kernel's matrix-core path for grouped queries holds
// (query head, group) pairs in the 16 rows of a tile.
bool layout_ok(const moqae_cfg *c) {
    if (c->chunk % 64 && c->chunk != 32 && c->chunk != 16 && c->chunk != 8) return false;
    const int rep = c->n_q_heads / c->n_kv_heads;
    return rep == 1 || rep * (kD / c->group) <= 16;
}
// Decode calls: keys quantised per channel are read by the single-head kernel only.
bool decode_ok(const moqae_cfg *c) { return layout_ok(c) && (!c->k_per_channel || c->n_q_heads == c->n_kv_heads); }

int first_16bit(const moqae_cfg *c) {
    for (int j = 0; j < c->n_experts; j++) if (c->expert_bits[j] == 16) return j;
    return -1;
}

bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

bool strides_ok(const moqae_cfg *c, int64_t sb, int64_t sh, int64_t ss) {
    (void)c;
    return ss >= kD && ss % 8 == 0 && sb % 8 == 0 && sh % 8 == 0 && sb >= 0 && sh >= 0;
}

int cu_count() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
        else cus = 256;                                                   // MI355X
    }
    return cus;
}

// Persistent workgroups of the decode kernel: one per compute unit (its eight wavefronts of up to 256
// registers and its LDS tables fill one), but never more than there are tickets of 128 tokens to hand to
// their wavefronts.  The only device query is the number of compute units of the current device.
int choose_wgs(const moqae_cfg *c, int n_chunks, int n_tail) {
    const int rep = c->n_q_heads / c->n_kv_heads;
    const int per_cu = 1;
    const int64_t rows = (int64_t)c->batch * c->n_kv_heads;
    const int64_t tickets = rows * ((int64_t)n_chunks * (c->chunk >= 256 ? c->chunk / 128 : 1) + (n_tail + 127) / 128);
    int64_t n = (int64_t)cu_count() * per_cu;
    const int64_t cap = (tickets + attn_waves_per_wg(rep) - 1) / attn_waves_per_wg(rep);
    if (n > cap) n = cap;
    if (n < 1) n = 1;
    return (int)n;
}

// Workspace: the ticket counters of the rows, then one partial (o[D], m, l) per query head and per
// workgroup that can touch its row.  Sized for the largest residual (n_tail = chunk - 1) so that it
// does not depend on n_tail.
uint64_t counters_bytes(const moqae_cfg *c, int n_chunks) {
    return ((uint64_t)attn_counter_bytes(c->batch * c->n_kv_heads, n_chunks, c->chunk) + 255u) & ~255ull;
}
uint64_t workspace_bytes(const moqae_cfg *c, int n_chunks) {
    const int BH = c->batch * c->n_kv_heads;
    const int n_wg = choose_wgs(c, n_chunks, c->chunk - 1);
    const uint64_t rows = (uint64_t)c->batch * c->n_q_heads;
    return counters_bytes(c, n_chunks) + rows * (uint64_t)attn_max_partials(n_wg, BH) * (kD + 2) * sizeof(float);
}
// Ragged batches: one long sequence among short ones can meet every workgroup's interval.
uint64_t workspace_bytes_ragged(const moqae_cfg *c, int max_chunks) {
    const int n_wg = choose_wgs(c, max_chunks, c->chunk - 1);
    const uint64_t rows = (uint64_t)c->batch * c->n_q_heads;
    return counters_bytes(c, max_chunks) + rows * (uint64_t)n_wg * (kD + 2) * sizeof(float);
}

// Device address of `scratch` on every GPU, looked up once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOQAE_E_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MOQAE_E_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MOQAE_OK;
}

// Geometry of the paged store from the configuration: page sizes, pool bases, ring positions.
bool pool_cfg_ok(const moqae_cfg *c, const moqae_pool_cfg *pc) {
    if (!pc) return false;
    uint64_t pages = 0;
    for (int j = 0; j < c->n_experts; j++) { if (pc->n_pages[j] < 0) return false; pages += (uint64_t)pc->n_pages[j]; }
    return pages < (1ull << 30);
}
uint64_t page_bytes_of(const moqae_cfg *c, int j) { return (block_bytes(c->chunk, c->group, c->expert_bits[j]) + 255u) & ~255ull; }
void fill_pool_geometry(const moqae_cfg *c, const moqae_pool_cfg *pc, PagedArgs &a) {
    uint64_t base = 0; uint32_t ring = 16 + 8 * 2 * kPoolShards;
    for (int j = 0; j < 8; j++) {
        const bool on = j < c->n_experts;
        a.n_pages[j] = on ? (uint32_t)pc->n_pages[j] : 0u;
        a.page_bytes[j] = on ? (uint32_t)page_bytes_of(c, j) : 0u;
        a.pool_base[j] = base; a.ring_start[j] = ring;
        a.ring_cap[j] = (a.n_pages[j] + kPoolShards - 1) / kPoolShards; if (a.ring_cap[j] == 0) a.ring_cap[j] = 1;
        a.bits_of[j] = on ? c->expert_bits[j] : 16;
        base += (uint64_t)a.n_pages[j] * a.page_bytes[j]; ring += on ? a.ring_cap[j] * kPoolShards : 0u;
    }
    a.M = c->n_experts; a.N = c->chunk; a.G = c->group; a.Hkv = c->n_kv_heads; a.BH = c->batch * c->n_kv_heads;
    a.kpc = c->k_per_channel;
}

thread_local hipEvent_t g_time_begin = nullptr, g_time_end = nullptr;   // measurement aid, see moqae_bench.h

}  // namespace

extern "C" {

int moqae_bench_time_decode_kernel(void *event_begin, void *event_end) {
    g_time_begin = static_cast<hipEvent_t>(event_begin); g_time_end = static_cast<hipEvent_t>(event_end);
    return MOQAE_OK;
}

uint32_t moqae_abi_version(void) { return MOQAE_ABI_VERSION; }

const char *moqae_strerror(int code) {
    switch (code) {
        case MOQAE_OK: return "ok";
        case MOQAE_E_INVAL: return "invalid argument or configuration";
        case MOQAE_E_WORKSPACE: return "decode workspace too small";
        case MOQAE_E_ARENA: return "packed arena too small";
        case MOQAE_E_HIP: return "HIP call or kernel launch failed";
    }
    return "unknown error";
}

uint64_t moqae_chunk_block_bytes(const moqae_cfg *cfg, int32_t bits) {
    if (!cfg_ok(cfg) || !bits_ok(bits)) return 0;
    return block_bytes(cfg->chunk, cfg->group, bits);
}

uint64_t moqae_arena_upper_bound(const moqae_cfg *cfg, int64_t n_chunks_total) {
    if (!cfg_ok(cfg) || n_chunks_total < 0) return 0;
    return 256u + (uint64_t)n_chunks_total * ((block_bytes(cfg->chunk, cfg->group, 16) + 255u) & ~255ull);
}

uint64_t moqae_decode_workspace_bytes(const moqae_cfg *cfg, int32_t n_chunks) {
    if (!cfg_ok(cfg) || !layout_ok(cfg) || n_chunks < 0) return 0;
    return workspace_bytes(cfg, n_chunks);
}

int moqae_route_chunks(const moqae_cfg *cfg,
                       const void *K, int64_t stride_b, int64_t stride_h, int64_t stride_s,
                       int32_t chunk_begin, int32_t chunk_end,
                       const void *W1, const void *W2, const void *W3,
                       const float *logit_bias,
                       uint8_t *expert, int64_t expert_stride,
                       int32_t *votes,
                       void *stream) {
    if (!cfg_ok(cfg) || !K || !W1 || !W2 || !W3 || !expert) return MOQAE_E_INVAL;
    if (chunk_begin < 0 || chunk_end < chunk_begin || expert_stride < chunk_end) return MOQAE_E_INVAL;
    if (!strides_ok(cfg, stride_b, stride_h, stride_s) || !aligned(K, 16)) return MOQAE_E_INVAL;
    if (!aligned(W1, 4) || !aligned(W2, 4) || !aligned(W3, 2)) return MOQAE_E_INVAL;
    const int e16 = first_16bit(cfg);
    if (cfg->freeze_chunks > 0 && e16 < 0) return MOQAE_E_INVAL;
    if (chunk_end == chunk_begin) return MOQAE_OK;

    RouteArgs a;
    a.K = static_cast<const uint16_t *>(K); a.stride_b = stride_b; a.stride_h = stride_h; a.stride_s = stride_s;
    a.W1 = static_cast<const uint16_t *>(W1); a.W2 = static_cast<const uint16_t *>(W2);
    a.W3 = static_cast<const uint16_t *>(W3); a.bias = logit_bias;
    a.expert = expert; a.expert_stride = expert_stride; a.votes = votes;
    a.chunk_begin = chunk_begin; a.N = cfg->chunk; a.Hkv = cfg->n_kv_heads;
    a.freeze_chunks = cfg->freeze_chunks; a.e16 = e16 < 0 ? 0 : e16;
    hipError_t e = launch_route(a, cfg->n_experts, chunk_end - chunk_begin, cfg->batch * cfg->n_kv_heads,
                                static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

int moqae_quantize_pack(const moqae_cfg *cfg,
                        const void *K, const void *V,
                        int64_t stride_b, int64_t stride_h, int64_t stride_s,
                        int32_t chunk_begin, int32_t chunk_end,
                        const uint8_t *expert, int64_t expert_stride,
                        void *arena, uint64_t arena_capacity,
                        uint64_t *arena_used,
                        uint64_t *chunk_off, int64_t off_stride,
                        int32_t *status,
                        void *stream) {
    if (!cfg_ok(cfg) || !layout_ok(cfg) || !K || !V || !expert || !arena || !arena_used || !chunk_off || !status) return MOQAE_E_INVAL;
    if (chunk_begin < 0 || chunk_end < chunk_begin) return MOQAE_E_INVAL;
    if (chunk_end - chunk_begin > 65535) return MOQAE_E_INVAL;             // grid.y of the pack kernel
    if (expert_stride < chunk_end || off_stride < chunk_end) return MOQAE_E_INVAL;
    if (!strides_ok(cfg, stride_b, stride_h, stride_s) || !aligned(K, 16) || !aligned(V, 16)) return MOQAE_E_INVAL;
    if (!aligned(arena, 256) || !aligned(arena_used, 8) || !aligned(chunk_off, 8) || !aligned(status, 4)) return MOQAE_E_INVAL;
    if (chunk_end == chunk_begin) return MOQAE_OK;

    PackArgs a;
    a.K = static_cast<const uint16_t *>(K); a.V = static_cast<const uint16_t *>(V);
    a.stride_b = stride_b; a.stride_h = stride_h; a.stride_s = stride_s;
    a.expert = expert; a.expert_stride = expert_stride;
    a.arena = static_cast<uint8_t *>(arena); a.capacity = arena_capacity; a.arena_used = arena_used;
    a.chunk_off = chunk_off; a.off_stride = off_stride; a.status = status;
    a.chunk_begin = chunk_begin; a.n_chunks = chunk_end - chunk_begin;
    a.BH = cfg->batch * cfg->n_kv_heads; a.N = cfg->chunk; a.G = cfg->group; a.Hkv = cfg->n_kv_heads;
    a.M = cfg->n_experts; a.kpc = cfg->k_per_channel;
    for (int j = 0; j < 8; j++) a.bits_of[j] = j < cfg->n_experts ? cfg->expert_bits[j] : 16;
    hipError_t e = launch_pack(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

static int decode_uniform(const moqae_cfg *cfg,
                          const void *q,
                          const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                          int64_t desc_stride, int32_t n_chunks,
                          const void *K_tail, const void *V_tail, int32_t n_tail,
                          float softmax_scale,
                          float *out,
                          void *workspace, uint64_t workspace_bytes,
                          void *stream, int planned, int nq = 1) {
    if (!cfg_ok(cfg) || !decode_ok(cfg) || !q || !out || !workspace) return MOQAE_E_INVAL;
    if (n_chunks < 0 || n_tail < 0 || n_tail >= cfg->chunk || n_chunks + n_tail <= 0) return MOQAE_E_INVAL;
    if (n_chunks > 0 && (!arena || !chunk_off || !expert || desc_stride < n_chunks)) return MOQAE_E_INVAL;
    if (n_tail > 0 && (!K_tail || !V_tail)) return MOQAE_E_INVAL;
    if (!aligned(q, 4) || !aligned(out, 8) || !aligned(workspace, 256)) return MOQAE_E_INVAL;
    if (n_chunks > 0 && (!aligned(arena, 256) || !aligned(chunk_off, 8))) return MOQAE_E_INVAL;
    if (n_tail > 0 && (!aligned(K_tail, 16) || !aligned(V_tail, 16))) return MOQAE_E_INVAL;
    if (workspace_bytes < moqae_decode_workspace_bytes(cfg, n_chunks)) return MOQAE_E_WORKSPACE;

    AttnArgs a;
    a.q = static_cast<const uint16_t *>(q); a.arena = static_cast<const uint8_t *>(arena);
    a.chunk_off = chunk_off; a.expert = expert; a.desc_stride = desc_stride;
    a.K_tail = static_cast<const uint16_t *>(K_tail); a.V_tail = static_cast<const uint16_t *>(V_tail);
    a.seq_chunks = nullptr; a.seq_tail = nullptr; a.planned = planned; a.kpc = cfg->k_per_channel;
    a.nq = nq; a.rep_in = cfg->n_q_heads / cfg->n_kv_heads / nq;
    a.counters = static_cast<unsigned int *>(workspace);
    a.part = reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) + counters_bytes(cfg, n_chunks)); a.out = out;
    a.scale_log2 = softmax_scale * 1.4426950408889634f;
    a.n_chunks = n_chunks; a.n_tail = n_tail;
    a.n_wg = choose_wgs(cfg, n_chunks, n_tail);
    a.max_partials = attn_max_partials(a.n_wg, cfg->batch * cfg->n_kv_heads);
    a.N = cfg->chunk; a.G = cfg->group; a.Hkv = cfg->n_kv_heads; a.rep = cfg->n_q_heads / cfg->n_kv_heads;
    a.BH = cfg->batch * cfg->n_kv_heads;
    for (int j = 0; j < 8; j++) a.bits_of[j] = j < cfg->n_experts ? cfg->expert_bits[j] : 16;
    hipError_t e = launch_attn(a, static_cast<hipStream_t>(stream), g_time_begin, g_time_end);
    return e == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

int moqae_append_tail(const moqae_cfg *cfg, const void *k_new, const void *v_new, void *K_tail, void *V_tail,
                      int32_t n_tail, void *stream) {
    if (!cfg_ok(cfg) || !layout_ok(cfg) || !k_new || !v_new || !K_tail || !V_tail) return MOQAE_E_INVAL;
    if (n_tail < 0 || n_tail >= cfg->chunk) return MOQAE_E_INVAL;
    if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(K_tail, 16) || !aligned(V_tail, 16)) return MOQAE_E_INVAL;
    hipError_t e = launch_append_tail(k_new, v_new, K_tail, V_tail, cfg->batch * cfg->n_kv_heads, cfg->chunk, n_tail,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

int moqae_decode_attn(const moqae_cfg *cfg, const void *q,
                      const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                      int64_t desc_stride, int32_t n_chunks,
                      const void *K_tail, const void *V_tail, int32_t n_tail,
                      float softmax_scale, float *out, void *workspace, uint64_t workspace_bytes, void *stream) {
    return decode_uniform(cfg, q, arena, chunk_off, expert, desc_stride, n_chunks, K_tail, V_tail, n_tail, softmax_scale,
                          out, workspace, workspace_bytes, stream, 0);
}

int moqae_decode_attn_static(const moqae_cfg *cfg, const void *q,
                             const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                             int64_t desc_stride, int32_t n_chunks,
                             const void *K_tail, const void *V_tail, int32_t n_tail,
                             float softmax_scale, float *out, void *stream) {
    if (!cfg_ok(cfg) || !layout_ok(cfg) || n_chunks < 0) return MOQAE_E_INVAL;
    if (workspace_bytes(cfg, n_chunks) > (uint64_t)MOQAE_STATIC_SCRATCH_BYTES) return MOQAE_E_WORKSPACE;
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != MOQAE_OK) return rc;
    return decode_uniform(cfg, q, arena, chunk_off, expert, desc_stride, n_chunks, K_tail, V_tail, n_tail, softmax_scale,
                          out, ws, MOQAE_STATIC_SCRATCH_BYTES, stream, 0);
}

uint64_t moqae_static_scratch_bytes(void) { return MOQAE_STATIC_SCRATCH_BYTES; }

uint64_t moqae_pool_page_bytes(const moqae_cfg *cfg, int32_t expert) {
    if (!cfg_ok(cfg) || expert < 0 || expert >= cfg->n_experts) return 0;
    return page_bytes_of(cfg, expert);
}
uint64_t moqae_pool_base(const moqae_cfg *cfg, const moqae_pool_cfg *pool, int32_t expert) {
    if (!cfg_ok(cfg) || !pool_cfg_ok(cfg, pool) || expert < 0 || expert > cfg->n_experts) return 0;
    PagedArgs a = {}; fill_pool_geometry(cfg, pool, a);
    return expert == cfg->n_experts ? a.pool_base[expert - 1] + (uint64_t)a.n_pages[expert - 1] * a.page_bytes[expert - 1]
                                    : a.pool_base[expert];
}
uint64_t moqae_pool_arena_bytes(const moqae_cfg *cfg, const moqae_pool_cfg *pool) { return moqae_pool_base(cfg, pool, cfg ? cfg->n_experts : 0); }
uint64_t moqae_pool_state_bytes(const moqae_cfg *cfg, const moqae_pool_cfg *pool) {
    if (!cfg_ok(cfg) || !pool_cfg_ok(cfg, pool)) return 0;
    PagedArgs a = {}; fill_pool_geometry(cfg, pool, a);
    const int last = cfg->n_experts - 1;
    return 4ull * (a.ring_start[last] + (uint64_t)a.ring_cap[last] * kPoolShards);
}

int moqae_pool_free_pages(const moqae_cfg *cfg, const moqae_pool_cfg *pool, const void *state, uint32_t *counts, void *stream) {
    if (!cfg_ok(cfg) || !pool_cfg_ok(cfg, pool) || !state || !counts || !aligned(state, 4) || !aligned(counts, 4)) return MOQAE_E_INVAL;
    PagedArgs a = {}; fill_pool_geometry(cfg, pool, a);
    a.state = static_cast<uint32_t *>(const_cast<void *>(state));
    return launch_pool_free_pages(a, counts, static_cast<hipStream_t>(stream)) == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

int moqae_pool_init(const moqae_cfg *cfg, const moqae_pool_cfg *pool, void *state, void *stream) {
    if (!cfg_ok(cfg) || !pool_cfg_ok(cfg, pool) || !state || !aligned(state, 4)) return MOQAE_E_INVAL;
    PagedArgs a = {}; fill_pool_geometry(cfg, pool, a);
    a.state = static_cast<uint32_t *>(state);
    return launch_pool_init(a, static_cast<hipStream_t>(stream)) == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

int moqae_route_pack_paged(const moqae_cfg *cfg, const moqae_pool_cfg *pool,
                           const void *K, const void *V, int64_t stride_b, int64_t stride_h, int64_t stride_s,
                           int32_t chunk_begin, int32_t chunk_end,
                           const void *W1, const void *W2, const void *W3, const float *logit_bias,
                           uint8_t *expert, int64_t expert_stride, int32_t *votes,
                           void *arena, void *state, uint64_t *chunk_off, int64_t off_stride, int32_t *status, void *stream) {
    if (!cfg_ok(cfg) || !layout_ok(cfg) || !pool_cfg_ok(cfg, pool) || !K || !V || !expert || !arena || !state || !chunk_off || !status)
        return MOQAE_E_INVAL;
    if (chunk_begin < 0 || chunk_end < chunk_begin || chunk_end - chunk_begin > 65535) return MOQAE_E_INVAL;
    if (expert_stride < chunk_end || off_stride < chunk_end) return MOQAE_E_INVAL;
    if (!strides_ok(cfg, stride_b, stride_h, stride_s) || !aligned(K, 16) || !aligned(V, 16)) return MOQAE_E_INVAL;
    if (!aligned(arena, 256) || !aligned(state, 4) || !aligned(chunk_off, 8) || !aligned(status, 4)) return MOQAE_E_INVAL;
    if (W1 && (!W2 || !W3 || !aligned(W1, 4) || !aligned(W2, 4) || !aligned(W3, 2))) return MOQAE_E_INVAL;
    const int e16 = first_16bit(cfg);
    if (W1 && cfg->freeze_chunks > 0 && e16 < 0) return MOQAE_E_INVAL;
    if (chunk_end == chunk_begin) return MOQAE_OK;
    PagedArgs a = {}; fill_pool_geometry(cfg, pool, a);
    a.K = static_cast<const uint16_t *>(K); a.V = static_cast<const uint16_t *>(V);
    a.stride_b = stride_b; a.stride_h = stride_h; a.stride_s = stride_s;
    a.W1 = static_cast<const uint16_t *>(W1); a.W2 = static_cast<const uint16_t *>(W2); a.W3 = static_cast<const uint16_t *>(W3);
    a.bias = logit_bias; a.expert = expert; a.expert_stride = expert_stride; a.votes = votes;
    a.arena = static_cast<uint8_t *>(arena); a.state = static_cast<uint32_t *>(state);
    a.chunk_off = reinterpret_cast<unsigned long long *>(chunk_off); a.off_stride = off_stride; a.status = status;
    a.chunk_begin = chunk_begin; a.n_chunks = chunk_end - chunk_begin;
    a.freeze_chunks = cfg->freeze_chunks; a.e16 = e16 < 0 ? 0 : e16;
    return launch_route_pack_paged(a, static_cast<hipStream_t>(stream)) == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

int moqae_pool_release(const moqae_cfg *cfg, const moqae_pool_cfg *pool,
                       const uint8_t *expert, int64_t expert_stride, uint64_t *chunk_off, int64_t off_stride,
                       int32_t row_begin, int32_t row_end, int32_t chunk_begin, int32_t chunk_end, void *state, void *stream) {
    if (!cfg_ok(cfg) || !pool_cfg_ok(cfg, pool) || !expert || !chunk_off || !state) return MOQAE_E_INVAL;
    if (row_begin < 0 || row_end < row_begin || row_end > cfg->batch * cfg->n_kv_heads) return MOQAE_E_INVAL;
    if (chunk_begin < 0 || chunk_end < chunk_begin || expert_stride < chunk_end || off_stride < chunk_end) return MOQAE_E_INVAL;
    if (!aligned(state, 4) || !aligned(chunk_off, 8)) return MOQAE_E_INVAL;
    PagedArgs a = {}; fill_pool_geometry(cfg, pool, a);
    a.expert = const_cast<uint8_t *>(expert); a.expert_stride = expert_stride;
    a.chunk_off = reinterpret_cast<unsigned long long *>(chunk_off); a.off_stride = off_stride;
    a.state = static_cast<uint32_t *>(state);
    a.chunk_begin = chunk_begin; a.n_chunks = chunk_end - chunk_begin;
    return launch_pool_release(a, row_begin, row_end - row_begin, static_cast<hipStream_t>(stream)) == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

int moqae_router_loss_grad(const moqae_cfg *cfg,
                           const void *K, int64_t stride_b, int64_t stride_h, int64_t stride_s,
                           int32_t token_begin, int32_t token_end,
                           const void *W1, const void *W2, const void *W3, const float *logit_bias,
                           const float *nll, const float *penalty_model, const float *penalty_mem, float lambda,
                           float *loss, float *dW1, float *dW2, float *dW3, float *dbias, void *stream) {
    if (!cfg_ok(cfg) || !K || !W1 || !W2 || !W3 || !nll || !loss || !dW1 || !dW2 || !dW3) return MOQAE_E_INVAL;
    if (token_begin < 0 || token_end <= token_begin) return MOQAE_E_INVAL;
    if (!strides_ok(cfg, stride_b, stride_h, stride_s) || !aligned(K, 16)) return MOQAE_E_INVAL;
    if (!aligned(W1, 4) || !aligned(W2, 4) || !aligned(W3, 2) || !aligned(nll, 4) || !aligned(loss, 4)) return MOQAE_E_INVAL;
    if (!aligned(dW1, 4) || !aligned(dW2, 4) || !aligned(dW3, 4) || !aligned(dbias, 4)) return MOQAE_E_INVAL;
    TrainArgs a = {};
    a.K = static_cast<const uint16_t *>(K); a.stride_b = stride_b; a.stride_h = stride_h; a.stride_s = stride_s;
    a.W1 = static_cast<const uint16_t *>(W1); a.W2 = static_cast<const uint16_t *>(W2); a.W3 = static_cast<const uint16_t *>(W3);
    a.bias = logit_bias; a.nll = nll;
    for (int j = 0; j < 8; j++) {                         // defaults: the penalties as Eq. (3) and Eq. (4) print them
        const float bj = j < cfg->n_experts ? (float)cfg->expert_bits[j] : 16.0f;
        a.pen_model[j] = (penalty_model && j < cfg->n_experts) ? penalty_model[j] : 1.0f / bj;
        a.pen_mem[j] = (penalty_mem && j < cfg->n_experts) ? penalty_mem[j] : 16.0f / bj;
    }
    a.lambda = lambda;
    a.token_begin = token_begin; a.n_tok = token_end - token_begin;
    a.BH = cfg->batch * cfg->n_kv_heads; a.Hkv = cfg->n_kv_heads; a.M = cfg->n_experts;
    a.inv_T = (float)(1.0 / ((double)a.BH * (double)a.n_tok));
    a.loss3 = loss; a.dW1 = dW1; a.dW2 = dW2; a.dW3 = dW3; a.dbias = dbias;
    return launch_router_train(a, cu_count(), static_cast<hipStream_t>(stream)) == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

int moqae_decode_attn_multi(const moqae_cfg *cfg, const void *q, int32_t n_queries,
                            const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                            int64_t desc_stride, int32_t n_chunks,
                            const void *K_tail, const void *V_tail, int32_t n_tail,
                            float softmax_scale, float *out, void *workspace, uint64_t workspace_bytes, void *stream) {
    if (!cfg_ok(cfg) || n_queries < 1 || n_queries > 8 || n_tail < n_queries) return MOQAE_E_INVAL;
    moqae_cfg c2 = *cfg;                                  // the queries of a KV head: n_queries * Hq / Hkv rows of the kernel's tile
    c2.n_q_heads = cfg->n_q_heads * n_queries;
    return decode_uniform(&c2, q, arena, chunk_off, expert, desc_stride, n_chunks, K_tail, V_tail, n_tail, softmax_scale,
                          out, workspace, workspace_bytes, stream, 0, n_queries);
}
uint64_t moqae_decode_workspace_bytes_multi(const moqae_cfg *cfg, int32_t n_chunks, int32_t n_queries) {
    if (!cfg_ok(cfg) || n_queries < 1 || n_queries > 8 || n_chunks < 0) return 0;
    moqae_cfg c2 = *cfg;
    c2.n_q_heads = cfg->n_q_heads * n_queries;
    return moqae_decode_workspace_bytes(&c2, n_chunks);
}

int moqae_decode_attn_planned(const moqae_cfg *cfg, const void *q,
                              const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                              int64_t desc_stride, int32_t n_chunks,
                              const void *K_tail, const void *V_tail, int32_t n_tail,
                              float softmax_scale, float *out, void *workspace, uint64_t workspace_bytes, void *stream) {
    return decode_uniform(cfg, q, arena, chunk_off, expert, desc_stride, n_chunks, K_tail, V_tail, n_tail, softmax_scale,
                          out, workspace, workspace_bytes, stream, 1);
}

int moqae_decode_plan(const moqae_cfg *cfg, const uint8_t *expert, int64_t desc_stride, int32_t n_chunks,
                      void *workspace, uint64_t workspace_bytes, void *stream) {
    if (!cfg_ok(cfg) || !layout_ok(cfg) || !workspace || n_chunks < 0) return MOQAE_E_INVAL;
    if (n_chunks > 0 && (!expert || desc_stride < n_chunks)) return MOQAE_E_INVAL;
    if (!aligned(workspace, 256)) return MOQAE_E_INVAL;
    if (workspace_bytes < moqae_decode_workspace_bytes(cfg, n_chunks)) return MOQAE_E_WORKSPACE;
    AttnArgs a = {};
    a.expert = expert; a.desc_stride = desc_stride;
    a.counters = static_cast<unsigned int *>(workspace);
    a.n_chunks = n_chunks; a.n_tail = cfg->chunk / 2;
    a.N = cfg->chunk; a.G = cfg->group; a.Hkv = cfg->n_kv_heads; a.rep = cfg->n_q_heads / cfg->n_kv_heads;
    a.BH = cfg->batch * cfg->n_kv_heads;
    for (int j = 0; j < 8; j++) a.bits_of[j] = j < cfg->n_experts ? cfg->expert_bits[j] : 16;
    return launch_attn_plan(a, static_cast<hipStream_t>(stream)) == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

int moqae_decode_attn_ragged(const moqae_cfg *cfg,
                             const void *q,
                             const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                             int64_t desc_stride,
                             const int32_t *n_chunks_seq, int32_t max_chunks,
                             const void *K_tail, const void *V_tail, const int32_t *n_tail_seq,
                             float softmax_scale,
                             float *out,
                             void *workspace, uint64_t workspace_bytes,
                             void *stream) {
    if (!cfg_ok(cfg) || !decode_ok(cfg) || !q || !out || !workspace || !n_chunks_seq || !n_tail_seq) return MOQAE_E_INVAL;
    if (max_chunks < 0) return MOQAE_E_INVAL;
    if (max_chunks > 0 && (!arena || !chunk_off || !expert || desc_stride < max_chunks)) return MOQAE_E_INVAL;
    if (!K_tail || !V_tail) return MOQAE_E_INVAL;
    if (!aligned(q, 4) || !aligned(out, 8) || !aligned(workspace, 256)) return MOQAE_E_INVAL;
    if (!aligned(n_chunks_seq, 4) || !aligned(n_tail_seq, 4)) return MOQAE_E_INVAL;
    if (max_chunks > 0 && (!aligned(arena, 256) || !aligned(chunk_off, 8))) return MOQAE_E_INVAL;
    if (!aligned(K_tail, 16) || !aligned(V_tail, 16)) return MOQAE_E_INVAL;
    if (workspace_bytes < workspace_bytes_ragged(cfg, max_chunks)) return MOQAE_E_WORKSPACE;

    AttnArgs a;
    a.q = static_cast<const uint16_t *>(q); a.arena = static_cast<const uint8_t *>(arena);
    a.chunk_off = chunk_off; a.expert = expert; a.desc_stride = desc_stride;
    a.K_tail = static_cast<const uint16_t *>(K_tail); a.V_tail = static_cast<const uint16_t *>(V_tail);
    a.seq_chunks = n_chunks_seq; a.seq_tail = n_tail_seq; a.planned = 0; a.kpc = cfg->k_per_channel;
    a.nq = 1; a.rep_in = cfg->n_q_heads / cfg->n_kv_heads;
    a.counters = static_cast<unsigned int *>(workspace);
    a.part = reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) + counters_bytes(cfg, max_chunks)); a.out = out;
    a.scale_log2 = softmax_scale * 1.4426950408889634f;
    a.n_chunks = max_chunks; a.n_tail = cfg->chunk - 1;
    a.n_wg = choose_wgs(cfg, max_chunks, cfg->chunk - 1);
    a.max_partials = a.n_wg;
    a.N = cfg->chunk; a.G = cfg->group; a.Hkv = cfg->n_kv_heads; a.rep = cfg->n_q_heads / cfg->n_kv_heads;
    a.BH = cfg->batch * cfg->n_kv_heads;
    for (int j = 0; j < 8; j++) a.bits_of[j] = j < cfg->n_experts ? cfg->expert_bits[j] : 16;
    hipError_t e = launch_attn(a, static_cast<hipStream_t>(stream), g_time_begin, g_time_end);
    return e == hipSuccess ? MOQAE_OK : MOQAE_E_HIP;
}

uint64_t moqae_decode_workspace_bytes_ragged(const moqae_cfg *cfg, int32_t max_chunks) {
    if (!cfg_ok(cfg) || !layout_ok(cfg) || max_chunks < 0) return 0;
    return workspace_bytes_ragged(cfg, max_chunks);
}

}  // extern "C"
