/*
 * libmoqae -- MoQAE inference hot path on AMD MI355X (gfx950).
 *
 * Three operations (arXiv 2506.07533):
 *   moqae_route_chunks   chunk-wise routing of cached keys to bit-width experts
 *                        (router MLP Eq. (1), token top-1 + chunk majority vote
 *                        Eq. (2), Sec. 3.2; routing freezing, Sec. 3.4);
 *   moqae_quantize_pack  group-wise quantisation of every chunk at its routed
 *                        bit-width into a packed arena (Sec. 3.1: every chunk is
 *                        quantised at the bit-width its router chose; the
 *                        residual shorter than a chunk stays FP16, Sec. 3.2);
 *   moqae_decode_attn    single-token decode attention over the mixed-precision
 *                        cache with de-quantisation on the fly and a full-
 *                        precision softmax (Sec. "Limitations").
 * Routing sharing (Sec. 3.4) needs no entry point: a follower block passes its
 * group leader's `expert` table to moqae_quantize_pack.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer owned by the caller unless the comment
 *     says "host".  `cfg` is a host pointer, read during the call only.
 *   - Every call only enqueues work on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream): no allocation, no synchronisation.
 *   - Return value: MOQAE_OK or a negative MOQAE_E_* code.  Argument errors are
 *     detected on the host before anything is launched.
 *   - fp16 tensors are IEEE binary16; [B, Hkv, S, D] tensors are addressed by
 *     element strides with the last dimension contiguous.
 *
 * Packed chunk block (bit-width b, N tokens, D = head_dim, G = group):
 *   b < 16 : [K codes | K meta | V codes | V meta]
 *            codes area = N*D*b/8 bytes of little-endian 32-bit words (V codes of
 *            8-token chunks at 2 bits: twice that, see below), a word holds 32/b
 *            codes, the code with in-word index e sits at bit 16*(e%2) + b*(e/2);
 *            K codes: token-major rows of D*b/32 words, dim d -> word d/(32/b),
 *                     in-word index d%(32/b);
 *            V codes: dimension-major tiles of up to 64 slots x 4 words (1 KiB).
 *                     With TW = 32/b tokens per word, a slot holds a slice of
 *                     TQ = max(TW, 8) consecutive tokens of one dim (WD = TQ/TW
 *                     words) for CPK = 4/WD dims that lie 16 apart.  A token block
 *                     is TB = min(4*TQ, max(N, TQ)) tokens = QD = TB/TQ slices: QD = 4
 *                     for N >= 64; a shorter chunk is one block of QD = 1, 2 or 4
 *                     slices and a tile has 16*QD slots; 8 tokens at 2 bits fill half
 *                     of their one slice of 16 (the rest holds zero codes, so that
 *                     area has 16*D*2/8 bytes).  Token t: block t/TB, slice
 *                     qd = (t % TB)/TQ, word w = (t % TQ)/TW, in-word index t % TW.
 *                     Dim d = 16*ct + j: tile cg = ct/CPK of the block, slot
 *                     16*qd + j, word n = (ct % CPK)*WD + w; word index in the area =
 *                     ((block*D/(16*CPK) + cg)*16*QD + 16*qd + j)*4 + n;
 *            meta area = one 32-bit word per (token, group), token-major:
 *                     fp16 scale | fp16 zero << 16;  x^ = code*scale + zero.
 *   b = 16 : [K rows | V rows], raw fp16, token-major.
 * Quantiser (per token, per group of G consecutive dims): zero = min,
 *   scale = fp16 round-UP of (max-min)/(2^b-1) (1.0 if max == min),
 *   code = clamp(rint((x-zero) * (1/scale)), 0, 2^b-1), all in binary32 with
 *   round-to-nearest-even.  K and V must be finite fp16 values: an Inf or NaN
 *   in a group gives that group an Inf / NaN scale and undefined codes (the
 *   paper's method has no rule for them either).
 */
#ifndef MOQAE_H
#define MOQAE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOQAE_ABI_VERSION 2u
#define MOQAE_MAX_EXPERTS 8

enum {
    MOQAE_OK          =  0,
    MOQAE_E_INVAL     = -1,  /* bad configuration, null pointer, misalignment, bad range          */
    MOQAE_E_WORKSPACE = -2,  /* decode workspace smaller than moqae_decode_workspace_bytes()      */
    MOQAE_E_ARENA     = -3,  /* packed arena too small (reported through the device status word)  */
    MOQAE_E_HIP       = -4   /* a HIP call or kernel launch failed                                */
};

typedef struct {
    int32_t batch;          /* B                                                               */
    int32_t n_q_heads;      /* Hq;  Hq / Hkv must be 1, 2, 4 or 8 and, if > 1, (Hq/Hkv)*(D/G) <= 16;
                               query head hq reads KV head hq / (Hq/Hkv)                       */
    int32_t n_kv_heads;     /* Hkv                                                             */
    int32_t head_dim;       /* D, must be 128                                                  */
    int32_t chunk;          /* N tokens per chunk: 8, 16, 32 (the paper's default, Sec. 4.1; Table 3
                               sweeps 8..128) or a multiple of 64 up to 256 for pack and decode (the
                               V token blocks span 64 tokens at 2 bits); routing alone also takes
                               96, 160, 224                                                       */
    int32_t group;          /* G elements per quantisation group along D: 32 or 64             */
    int32_t n_experts;      /* M, 1..8                                                         */
    int32_t expert_bits[MOQAE_MAX_EXPERTS]; /* B_j in {2,4,8,16}; index order = tie-break order */
    int32_t freeze_chunks;  /* routing freezing (Sec. 3.4): chunks c < freeze_chunks are never
                               routed and take the first 16-bit expert; the paper uses 1       */
    int32_t k_per_channel;  /* 0: the keys' quantisation groups are G consecutive dims of a token
                               (as the values'); 1: G consecutive tokens of one dim (the outlier
                               channels of key caches, Sec. 2.2): needs N % G == 0; the K meta
                               area is then indexed [token group][dim], the codes keep their
                               places; decode attention: one query head per KV head, one
                               query per sequence (uniform and ragged calls alike)             */
} moqae_cfg;

/*
 * Router, Eq. (1)-(2) of Sec. 3.2, for chunks [chunk_begin, chunk_end) of every
 * (sequence b, KV head h).  Chunk c covers tokens [c*N, (c+1)*N) of K; token s
 * of (b, h) starts at K + b*stride_b + h*stride_h + s*stride_s (element
 * strides, stride_s a multiple of 8, base 16-byte aligned).
 *   logits = SiLU((x W1) * (x W2)) W3 (+ logit_bias), x = one cached key row;
 *   token expert = first arg-max of the logits; chunk expert = first arg-max of
 *   the per-expert token counts.  Evaluated in binary32, sums in index order,
 *   so the result is reproducible bit for bit.
 * W1, W2: fp16 [D, M] row-major; W3: fp16 [M, M] row-major (hidden j -> logit k
 * at W3[j*M+k]); logit_bias: fp32 [M] or NULL (Eq. (1) has none).
 * Out: expert[(b*Hkv+h)*expert_stride + c] = expert index;
 *      votes[((b*Hkv+h)*expert_stride + c)*M + k] = token count of expert k
 *      (all zero for frozen chunks); votes may be NULL.
 * Entries outside [chunk_begin, chunk_end) are not touched.
 * Errors: MOQAE_E_INVAL (also when freeze_chunks > 0 and no expert has 16 bits).
 */
int moqae_route_chunks(const moqae_cfg *cfg,
                       const void *K, int64_t stride_b, int64_t stride_h, int64_t stride_s,
                       int32_t chunk_begin, int32_t chunk_end,
                       const void *W1, const void *W2, const void *W3,
                       const float *logit_bias,
                       uint8_t *expert, int64_t expert_stride,
                       int32_t *votes,
                       void *stream);

/*
 * Quantise and pack chunks [chunk_begin, chunk_end) of every (b, h) of K and V
 * (same strides for both) at the bit-width of expert[...] (this block's own
 * decisions, or its routing-sharing leader's, Sec. 3.4).
 * Blocks are appended to `arena` in (b, h, c) order starting at *arena_used
 * rounded up to 256 bytes; each block start is 256-byte aligned;
 * chunk_off[(b*Hkv+h)*off_stride + c] receives the block's byte offset and
 * *arena_used the new end.  `arena` must be 256-byte aligned.  At most 65535
 * chunks per (sequence, KV head) and call (MOQAE_E_INVAL beyond; call again for more).
 * *status (device int32) must be 0 on entry, otherwise the call is a no-op; if
 * the blocks do not fit below arena_capacity, or an expert index is >= M,
 * *status becomes MOQAE_E_ARENA / MOQAE_E_INVAL and nothing else is written
 * (no arena byte, no offset, *arena_used unchanged).
 */
int moqae_quantize_pack(const moqae_cfg *cfg,
                        const void *K, const void *V,
                        int64_t stride_b, int64_t stride_h, int64_t stride_s,
                        int32_t chunk_begin, int32_t chunk_end,
                        const uint8_t *expert, int64_t expert_stride,
                        void *arena, uint64_t arena_capacity,
                        uint64_t *arena_used,
                        uint64_t *chunk_off, int64_t off_stride,
                        int32_t *status,
                        void *stream);

/*
 * Decode attention for one new token per sequence: for every query head,
 *   out = softmax(softmax_scale * q K^^T) V^
 * over the n_chunks packed chunks of its KV head followed by the n_tail FP16
 * residual rows (Sec. 3.2), with K^, V^ the de-quantised cache.  No mask: the
 * query attends to every cached token.
 * q: fp16 [B, Hq, D]; expert / chunk_off: the tables written by the two calls
 * above, row stride desc_stride (>= n_chunks); K_tail, V_tail: fp16
 * [B, Hkv, N, D] of which rows [0, n_tail) are valid, 0 <= n_tail < N (may be
 * NULL when n_tail == 0); n_chunks + n_tail must be > 0.
 * out: fp32 [B, Hq, D].  workspace: at least moqae_decode_workspace_bytes()
 * bytes, 256-byte aligned, contents irrelevant on entry (ticket counters and
 * the cost of every row, written by the first kernel of the call; one partial
 * softmax state per workgroup and row, merged by its last kernel).
 */
int moqae_decode_attn(const moqae_cfg *cfg,
                      const void *q,
                      const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                      int64_t desc_stride, int32_t n_chunks,
                      const void *K_tail, const void *V_tail, int32_t n_tail,
                      float softmax_scale,
                      float *out,
                      void *workspace, uint64_t workspace_bytes,
                      void *stream);

/*
 * The residual of Sec. 3.2 during decode: the new token's key and value rows (k_new, v_new: fp16 [B, Hkv, D],
 * contiguous) are written to row n_tail (0 <= n_tail < N) of the FP16 residual buffers K_tail, V_tail
 * (fp16 [B, Hkv, N, D], contiguous), which then hold n_tail + 1 valid rows.  All pointers 16-byte aligned.
 * When the residual reaches N rows the caller routes and packs it as the next chunk (moqae_route_chunks /
 * moqae_quantize_pack with the residual buffers as K, V) and starts again at row 0.
 */
int moqae_append_tail(const moqae_cfg *cfg, const void *k_new, const void *v_new, void *K_tail, void *V_tail,
                      int32_t n_tail, void *stream);

/*
 * Decode steps that follow one another on unchanged tables (routing decisions are made once when a chunk is
 * compressed and reused by every later decode step, Sec. 3.2 / 3.4): what the first kernel of moqae_decode_attn
 * derives from the tables -- the cost of every row, zeroed ticket counters -- is the same for all of them.
 * moqae_decode_plan leaves it in `workspace` (same size and alignment as for moqae_decode_attn);
 * moqae_decode_attn_planned is moqae_decode_attn without that first kernel: same arguments, same result, and it
 * leaves the plan in the workspace ready for the next call.  The plan holds as long as `expert`, desc_stride and
 * n_chunks do not change and nothing else writes the workspace; n_tail, q and the residual rows may change from
 * call to call.  After a chunk has been appended (moqae_quantize_pack), plan again.  Calls that share a workspace
 * must not overlap.
 */
int moqae_decode_plan(const moqae_cfg *cfg, const uint8_t *expert, int64_t desc_stride, int32_t n_chunks,
                      void *workspace, uint64_t workspace_bytes, void *stream);
int moqae_decode_attn_planned(const moqae_cfg *cfg,
                              const void *q,
                              const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                              int64_t desc_stride, int32_t n_chunks,
                              const void *K_tail, const void *V_tail, int32_t n_tail,
                              float softmax_scale,
                              float *out,
                              void *workspace, uint64_t workspace_bytes,
                              void *stream);

/*
 * The same attention for a batch whose sequences have different lengths (the residual rule of Sec. 3.2
 * applies per sequence: each keeps its own last S mod N tokens in FP16, so a batch served together ends
 * up with different numbers of packed chunks and of residual rows).
 * n_chunks_seq, n_tail_seq: DEVICE int32 [B], read by the kernels of the call: sequence b attends to its
 * first n_chunks_seq[b] packed chunks (<= max_chunks, values outside [0, max_chunks] are clamped) and to
 * the first n_tail_seq[b] rows of its residual (clamped to [0, N-1]).  A sequence with neither gets
 * zeros in `out`.  max_chunks (host) bounds the chunk counts and sizes the workspace; the tables' row
 * stride desc_stride must be >= max_chunks.  K_tail, V_tail must not be NULL.  Everything else as in
 * moqae_decode_attn; workspace: at least moqae_decode_workspace_bytes_ragged(cfg, max_chunks) bytes
 * (larger than the uniform call's: one long sequence among short ones can be shared by all workgroups).
 */
int moqae_decode_attn_ragged(const moqae_cfg *cfg,
                             const void *q,
                             const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                             int64_t desc_stride,
                             const int32_t *n_chunks_seq, int32_t max_chunks,
                             const void *K_tail, const void *V_tail, const int32_t *n_tail_seq,
                             float softmax_scale,
                             float *out,
                             void *workspace, uint64_t workspace_bytes,
                             void *stream);
uint64_t moqae_decode_workspace_bytes_ragged(const moqae_cfg *cfg, int32_t max_chunks);   /* host; 0 if cfg invalid */

/*
 * Several new tokens per sequence in one call (speculative decoding, chunked prefill) over the same packed cache:
 * q, out: [B, n_queries, Hq, D].  The new tokens' own K, V rows must already be the LAST n_queries valid rows of the
 * FP16 residual (n_tail >= n_queries); query t (0-based) attends to every packed chunk and to the first
 * n_tail - (n_queries - 1 - t) residual rows, i.e. causally among the new tokens.  n_queries * Hq / Hkv must be 1, 2,
 * 4 or 8 (and, above 1, times D/G at most 16): the queries of a KV head share every byte read, as grouped query heads
 * do.  Everything else as moqae_decode_attn; workspace: moqae_decode_workspace_bytes_multi(cfg, n_chunks, n_queries).
 */
int moqae_decode_attn_multi(const moqae_cfg *cfg,
                            const void *q, int32_t n_queries,
                            const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                            int64_t desc_stride, int32_t n_chunks,
                            const void *K_tail, const void *V_tail, int32_t n_tail,
                            float softmax_scale,
                            float *out,
                            void *workspace, uint64_t workspace_bytes,
                            void *stream);
uint64_t moqae_decode_workspace_bytes_multi(const moqae_cfg *cfg, int32_t n_chunks, int32_t n_queries);  /* host; 0 if invalid */

/*
 * Router fine-tuning, Sec. 3.3: the loss of Eq. (3)-(5) and its gradient with respect to the router weights, over
 * the cached key rows [token_begin, token_end) of every (b, h) (T rows in all), with the language model frozen:
 *   L_model = (1/T) sum_i p^i_j * L_nll * penalty_model[j],   L_mem = (1/T) sum_i p^i_j * penalty_mem[j],
 *   L = lambda * L_model + (1 - lambda) * L_mem,
 * where p^i = softmax of the logits of row i (Eq. (1)), j = its top-1 expert (the routing decision, taken in the
 * same binary32 arithmetic as moqae_route_chunks), and L_nll = nll[b], the frozen model's loss of the row's
 * sequence (device fp32 [B]; an input, here synthetic).  penalty_model, penalty_mem: HOST fp32 [M], or NULL for
 * the values Eq. (3) and Eq. (4) print, 1/B_j and 16/B_j (the text under Eq. (4) describes its penalty as the
 * inverse of Eq. (3)'s, which B_j/16 would be: pass it explicitly if that is wanted).
 * Out (device fp32, overwritten): loss[3] = L, L_model, L_mem; dW1, dW2 [D, M]; dW3 [M, M]; dbias [M] or NULL.
 * Evaluated in binary32; sums over rows are added in no fixed order (results agree to rounding, not bit for bit).
 */
int moqae_router_loss_grad(const moqae_cfg *cfg,
                           const void *K, int64_t stride_b, int64_t stride_h, int64_t stride_s,
                           int32_t token_begin, int32_t token_end,
                           const void *W1, const void *W2, const void *W3, const float *logit_bias,
                           const float *nll, const float *penalty_model, const float *penalty_mem, float lambda,
                           float *loss, float *dW1, float *dW2, float *dW3, float *dbias,
                           void *stream);

/*
 * Paged store.  The ordered arena of moqae_quantize_pack puts a chunk's block where the blocks of all earlier
 * chunks end, so nothing can be packed before every chunk of the call is routed, and nothing can ever be given
 * back.  Here every expert has a pool of equal pages instead: pool j = n_pages[j] pages of
 * moqae_pool_page_bytes(cfg, j) bytes (the expert's chunk block rounded up to 256), pool after pool in `arena`
 * (moqae_pool_base; moqae_pool_arena_bytes in all, 256-byte aligned).  The router (Eq. (1)-(2), Sec. 3.2),
 * the choice of a page and the quantiser then run in ONE pass over a chunk, which reads K from HBM once; the
 * blocks are the ones moqae_quantize_pack writes, and moqae_decode_attn* read them through `chunk_off` as before.
 * `state` (device, moqae_pool_state_bytes, 4-byte aligned) holds the free pages of every pool; its layout is the
 * library's own (the pages of a pool are spread over several rings, so that the atomic steps of a call do not
 * all meet on one address).  moqae_pool_init fills it (every page free); moqae_pool_free_pages writes the
 * number of free pages of every pool to counts[0..7] (device uint32).
 *
 * moqae_route_pack_paged, for chunks [chunk_begin, chunk_end) of every (b, h): W1 != NULL: routes the chunk as
 * moqae_route_chunks does (expert and votes are outputs; frozen chunks take the first 16-bit expert); W1 == NULL:
 * `expert` is an input (the decisions of a routing-sharing leader, Sec. 3.4) and votes is not touched.  Then a
 * page is taken from the expert's pool, chunk_off receives its byte offset and K, V are quantised into it.
 * Which page a chunk gets is not specified (any free page of the right pool).  *status (device int32) != 0 on
 * entry: nothing is done.  A chunk whose pool is empty gets chunk_off = ~0, is not packed, and *status becomes
 * MOQAE_E_ARENA (an expert index >= M given as input: MOQAE_E_INVAL); the other chunks of the call are still
 * served, and the caller must treat the call as failed.  At most 65535 chunks per (b, h) and call.
 *
 * moqae_pool_release gives the pages of chunks [chunk_begin, chunk_end) of rows [row_begin, row_end) (row =
 * b*Hkv + h) back to their pools and sets their chunk_off to ~0 (a finished sequence, the oldest chunks of a
 * sliding window); entries that are ~0 already are skipped.  Calls on one pool state must not overlap.
 */
typedef struct { int32_t n_pages[MOQAE_MAX_EXPERTS]; } moqae_pool_cfg;            /* pages of pool j = expert j */
uint64_t moqae_pool_page_bytes(const moqae_cfg *cfg, int32_t expert);                              /* host */
uint64_t moqae_pool_base(const moqae_cfg *cfg, const moqae_pool_cfg *pool, int32_t expert);       /* host */
uint64_t moqae_pool_arena_bytes(const moqae_cfg *cfg, const moqae_pool_cfg *pool);                /* host */
uint64_t moqae_pool_state_bytes(const moqae_cfg *cfg, const moqae_pool_cfg *pool);                /* host */
int moqae_pool_init(const moqae_cfg *cfg, const moqae_pool_cfg *pool, void *state, void *stream);
int moqae_pool_free_pages(const moqae_cfg *cfg, const moqae_pool_cfg *pool, const void *state, uint32_t *counts, void *stream);
int moqae_route_pack_paged(const moqae_cfg *cfg, const moqae_pool_cfg *pool,
                           const void *K, const void *V, int64_t stride_b, int64_t stride_h, int64_t stride_s,
                           int32_t chunk_begin, int32_t chunk_end,
                           const void *W1, const void *W2, const void *W3, const float *logit_bias,
                           uint8_t *expert, int64_t expert_stride, int32_t *votes,
                           void *arena, void *state, uint64_t *chunk_off, int64_t off_stride, int32_t *status,
                           void *stream);
int moqae_pool_release(const moqae_cfg *cfg, const moqae_pool_cfg *pool,
                       const uint8_t *expert, int64_t expert_stride, uint64_t *chunk_off, int64_t off_stride,
                       int32_t row_begin, int32_t row_end, int32_t chunk_begin, int32_t chunk_end,
                       void *state, void *stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): moqae_decode_attn without the workspace argument.  The workspace is a fixed array of
 * moqae_static_scratch_bytes() (8 MiB) that lives inside the library, one copy on every GPU the library is used
 * on, held until the process ends.  Same arguments otherwise, same result.  MOQAE_E_WORKSPACE if
 * moqae_decode_workspace_bytes(cfg, n_chunks) exceeds that size (e.g. batch * Hq above about 16 000 query rows);
 * nothing is launched then.  The call allocates nothing and frees nothing.  All calls on one GPU share the
 * array: calls that may overlap on one GPU (different streams, different threads) race and must be serialised
 * by the caller; nothing has to be cleared between calls.
 */
int moqae_decode_attn_static(const moqae_cfg *cfg,
                             const void *q,
                             const void *arena, const uint64_t *chunk_off, const uint8_t *expert,
                             int64_t desc_stride, int32_t n_chunks,
                             const void *K_tail, const void *V_tail, int32_t n_tail,
                             float softmax_scale,
                             float *out,
                             void *stream);
uint64_t moqae_static_scratch_bytes(void);                                       /* host */

/* Host helpers (no GPU work; moqae_decode_workspace_bytes* read the number of compute units of the current device). */
uint64_t moqae_chunk_block_bytes(const moqae_cfg *cfg, int32_t bits);            /* K+V block of one chunk; 0 if invalid */
uint64_t moqae_arena_upper_bound(const moqae_cfg *cfg, int64_t n_chunks_total);  /* all-16-bit worst case + alignment    */
uint64_t moqae_decode_workspace_bytes(const moqae_cfg *cfg, int32_t n_chunks);   /* 0 if cfg invalid                     */
const char *moqae_strerror(int code);
uint32_t moqae_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MOQAE_H */
