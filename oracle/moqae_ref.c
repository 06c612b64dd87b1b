/*
 * MoQAE inference hot path -- CPU ORACLE.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain statement of what
 * the GPU library must compute; only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table
 * or helper with the HIP implementation, and the product never falls back to
 * it.
 *
 * What comes from the paper (arXiv 2506.07533):
 *   - the router MLP, Eq. (1) of Sec. 3.2:  P = f(C W1 . C W2) W3 with f = SiLU
 *     (Sec. 4.1 "Implementation": SiLU, hidden size = number of experts, top-1);
 *   - token top-1 followed by the chunk majority vote, Eq. (2) of Sec. 3.2;
 *   - equal chunks of N tokens, the residual shorter than a chunk stays FP16
 *     (Sec. 3.2, first paragraph);
 *   - routing freezing: the first chunk never enters the router and is FP16
 *     (Sec. 3.4);
 *   - routing sharing needs no code here: a follower block is packed with the
 *     leader block's decisions (Sec. 3.4);
 *   - decode attention over the de-quantised cache with a high-precision
 *     softmax (Sec. "Limitations").
 * What the paper leaves open (quantiser formula, packed layout, tie rules,
 * the shape of W3) is fixed by this build's own specification; every such
 * reading is spelled out next to the code that takes it.
 *
 * Precision: routing and packing are defined in IEEE binary32 with one
 * rounding per written operation, in the written order (compile with
 * -ffp-contract=off, no fast-math), because their results are integers that
 * must be reproduced bit for bit.  Attention is the textbook definition in
 * binary64 over the decoded cache.
 *
 * Parity pins (tests/test_oracle_*.py): every function below is pinned to
 * something other than itself; see the list at the end of this header.
 *   half conversions   : exhaustive against numpy's float16
 *   exp_p              : against libm within 1e-5, exp_p(0) == 1, coefficients
 *                        equal (ln 2)^k / k! rounded to binary32
 *   route              : brute force of Eq. (1)-(2) in binary64, the one-hot
 *                        special case, vote invariants, constructed ties, RF
 *   quantise / pack    : hand-worked byte fixtures, round-trip bound scale/2,
 *                        constant groups, code range, bit-coverage bijection
 *   decode attention   : 16-bit experts == unquantised attention (torch fp64
 *                        scaled_dot_product_attention), S = 1, uniform keys,
 *                        score-shift invariance
 *   several queries    : an all-16-bit cache against torch fp64 attention with a causal
 *                        mask over the new tokens
 *   router loss (3)-(5): gradient against central finite differences of the loss
 *                        in binary64, one expert (p = 1: constant loss, zero
 *                        gradient), lambda = 0 / 1 limits, linearity in L_nll
 *   paged store        : pool sizes and bases by closed form; a set model of the
 *                        allocator written in the test (pages handed out in ring
 *                        order, given-back pages reused first-in first-out, no
 *                        page twice, exhaustion status); every page holds the
 *                        block the (pinned) chunk packer makes for its chunk
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t batch, n_q_heads, n_kv_heads, head_dim;
    int32_t chunk;          /* N tokens per chunk                                  */
    int32_t group;          /* G consecutive head-dim elements per quant group     */
    int32_t n_experts;      /* M                                                   */
    int32_t expert_bits[8]; /* bit-width B_j of expert j, each in {2,4,8,16}       */
    int32_t freeze_chunks;  /* RF: chunks c < freeze_chunks are FP16, never routed */
    int32_t k_per_channel;  /* 0: K groups = G consecutive dims of a token (as V);    */
                            /* 1: K groups = G consecutive tokens of one dim          */
} moqae_ref_cfg;

enum { REF_OK = 0, REF_E_INVAL = -1, REF_E_ARENA = -3 };

/* ------------------------------------------------------------------ */
/* binary16 <-> binary32, written out on the bit patterns (IEEE 754). */
/* ------------------------------------------------------------------ */

float moqae_ref_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    int32_t  e    = (h >> 10) & 0x1f;
    uint32_t frac = h & 0x3ffu;
    double v;
    if (e == 0)        v = ldexp((double)frac, -24);               /* zero / subnormal */
    else if (e == 31)  v = frac ? (double)NAN : (double)INFINITY;
    else               v = ldexp((double)(1024u + frac), e - 25);  /* (1+f/1024) 2^(e-15) */
    return (float)(sign ? -v : v);                                 /* exact: 11 bits fit */
}

/* round-to-nearest, ties-to-even */
uint16_t moqae_ref_float_to_half(float f)
{
    uint32_t u; memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    double a = fabs((double)f);
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);           /* rounds to inf */
    if (a == 0.0) return sign;
    int ex; (void)frexp(a, &ex);                                   /* a = m 2^ex, m in [0.5,1) */
    int e = ex - 1;                                                /* a = 1.x * 2^e */
    if (e < -14) e = -14;                                          /* subnormal quantum */
    double q = ldexp(a, 10 - e);                                   /* in units of one ulp */
    double r = nearbyint(q);                                       /* default mode: RNE */
    uint32_t m = (uint32_t)r;                                      /* 0 .. 2048 */
    uint32_t bits;
    if (e == -14 && m < 1024u) bits = m;                           /* subnormal (or zero) */
    else {
        if (m == 2048u) { m = 1024u; e += 1; }
        bits = ((uint32_t)(e + 15) << 10) | (m - 1024u);
    }
    return (uint16_t)(sign | bits);
}

#define H2F moqae_ref_half_to_float
#define F2H moqae_ref_float_to_half

/* ------------------------------------------------------------------ */
/* exp_p: the pinned exponential used by SiLU in the router.           */
/* 2^r on [-1/2, 1/2] by the degree-6 Taylor polynomial, Horner form,  */
/* every product and sum rounded separately to binary32.               */
/* ------------------------------------------------------------------ */

float moqae_ref_exp_p(float x)
{
    const float LOG2E = 0x1.715476p+0f;
    const float C1 = 0x1.62e430p-1f,  C2 = 0x1.ebfbe0p-3f,  C3 = 0x1.c6b08ep-5f;
    const float C4 = 0x1.3b2ab6p-7f,  C5 = 0x1.5d87fep-10f, C6 = 0x1.430912p-13f;
    if (x < -80.0f) x = -80.0f;
    if (x >  80.0f) x =  80.0f;
    float t = x * LOG2E;
    float n = rintf(t);
    float r = t - n;
    float p = C6;
    p = p * r; p = p + C5;
    p = p * r; p = p + C4;
    p = p * r; p = p + C3;
    p = p * r; p = p + C2;
    p = p * r; p = p + C1;
    p = p * r; p = p + 1.0f;
    uint32_t sb = (uint32_t)((int32_t)n + 127) << 23;              /* 2^n, n in [-116,116] */
    float s; memcpy(&s, &sb, 4);
    return p * s;
}

/* ------------------------------------------------------------------ */
/* helpers on the configuration                                        */
/* ------------------------------------------------------------------ */

static int bits_ok(int b) { return b == 2 || b == 4 || b == 8 || b == 16; }

static int cfg_ok(const moqae_ref_cfg *c)
{
    if (!c) return 0;
    if (c->batch < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1) return 0;
    if (c->n_q_heads % c->n_kv_heads) return 0;
    if (c->head_dim < 2 || c->head_dim % 2) return 0;
    if (c->group < 1 || c->head_dim % c->group) return 0;
    if (c->chunk != 8 && c->chunk != 16 && (c->chunk < 32 || c->chunk % 32)) return 0;
    if (c->n_experts < 1 || c->n_experts > 8) return 0;
    for (int j = 0; j < c->n_experts; j++) if (!bits_ok(c->expert_bits[j])) return 0;
    if (c->freeze_chunks < 0) return 0;
    if (c->k_per_channel != 0 && c->k_per_channel != 1) return 0;
    if (c->k_per_channel && c->chunk % c->group) return 0;        /* token groups must tile the chunk */
    return 1;
}

static int first_16bit_expert(const moqae_ref_cfg *c)
{
    for (int j = 0; j < c->n_experts; j++) if (c->expert_bits[j] == 16) return j;
    return -1;
}

/* Tokens the V code area has room for: the chunk's N, but at least one slice of the V layout
 * (see v_code_pos: max(32/b, 8) tokens), so a chunk of 8 tokens at 2 bits is stored as a slice
 * of 16 whose upper half holds zero codes.                                                    */
static int v_token_room(int N, int b)
{
    int TQ = 32 / b > 8 ? 32 / b : 8;
    return N < TQ ? TQ : N;
}

/* Bytes of one chunk block (K and V together) at bit-width b.
 * b < 16 : [K codes][K meta][V codes][V meta], K codes N*D*b/8 bytes, V codes
 *          v_token_room(N, b)*D*b/8 bytes, meta one 32-bit word per (token, group);
 * b = 16 : [K raw fp16][V raw fp16].                                  */
uint64_t moqae_ref_chunk_block_bytes(const moqae_ref_cfg *c, int32_t b)
{
    uint64_t N = (uint64_t)c->chunk, D = (uint64_t)c->head_dim, G = (uint64_t)c->group;
    if (b == 16) return 2u * N * D * 2u;
    return (N + (uint64_t)v_token_room(c->chunk, b)) * D * (uint64_t)b / 8u + 2u * N * (D / G) * 4u;
}

static uint64_t round_up_256(uint64_t x) { return (x + 255u) & ~(uint64_t)255u; }

/* ------------------------------------------------------------------ */
/* Router: Eq. (1) and Eq. (2) of Sec. 3.2, routing freezing Sec. 3.4. */
/*                                                                      */
/* Readings taken where the text is open:                               */
/*  - C is the chunk's N cached key rows of one KV head (D = per-head   */
/*    size, as the text under Eq. (1) says);                            */
/*  - "CW1 . CW2" is the element-wise product of two N x M matrices and */
/*    f is applied to that product;                                     */
/*  - W3 is M x M (the printed D x M cannot follow an N x M hidden      */
/*    layer; Sec. 4.1 gives the hidden size as the number of experts);  */
/*  - arg-max is taken on the logits (softmax is monotone); the first   */
/*    index wins every tie, for the token top-1 and for the vote;       */
/*  - an optional additive logit bias (not in Eq. (1); NULL = absent).  */
/* ------------------------------------------------------------------ */

/* logits of one token: x[D] (binary32 values of the fp16 row) -> p[M] */
static void router_token_logits(const float *x, int D, int M,
                                const float *w1, const float *w2, const float *w3,
                                const float *bias, float *p)
{
    float h[8];
    for (int m = 0; m < M; m++) {
        float a = 0.0f, b = 0.0f;
        for (int d = 0; d < D; d++) a = a + x[d] * w1[d * M + m];
        for (int d = 0; d < D; d++) b = b + x[d] * w2[d * M + m];
        float z = a * b;
        float e = moqae_ref_exp_p(-z);
        h[m] = z / (1.0f + e);                                     /* SiLU(z) = z * sigmoid(z) */
    }
    for (int k = 0; k < M; k++) {
        float acc = 0.0f;
        for (int j = 0; j < M; j++) acc = acc + h[j] * w3[j * M + k];
        if (bias) acc = acc + bias[k];
        p[k] = acc;
    }
}

int moqae_route_chunks_ref(const moqae_ref_cfg *cfg,
                           const uint16_t *K, int64_t stride_b, int64_t stride_h, int64_t stride_s,
                           int32_t chunk_begin, int32_t chunk_end,
                           const uint16_t *W1, const uint16_t *W2, const uint16_t *W3,
                           const float *logit_bias,
                           uint8_t *expert, int64_t expert_stride_bh,
                           int32_t *votes)
{
    if (!cfg_ok(cfg) || !K || !W1 || !W2 || !W3 || !expert) return REF_E_INVAL;
    if (chunk_begin < 0 || chunk_end < chunk_begin || expert_stride_bh < chunk_end) return REF_E_INVAL;
    const int D = cfg->head_dim, M = cfg->n_experts, N = cfg->chunk;
    const int e16 = first_16bit_expert(cfg);
    if (cfg->freeze_chunks > 0 && e16 < 0) return REF_E_INVAL;

    float *w1 = malloc(sizeof(float) * D * M), *w2 = malloc(sizeof(float) * D * M);
    float w3[64];
    for (int i = 0; i < D * M; i++) { w1[i] = H2F(W1[i]); w2[i] = H2F(W2[i]); }
    for (int i = 0; i < M * M; i++) w3[i] = H2F(W3[i]);

    const int64_t units = (int64_t)cfg->batch * cfg->n_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; u++) {
        const int64_t b = u / cfg->n_kv_heads, h = u % cfg->n_kv_heads;
        float *x = malloc(sizeof(float) * D);
        for (int c = chunk_begin; c < chunk_end; c++) {
            int32_t cnt[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            int best;
            if (c < cfg->freeze_chunks) {
                best = e16;                                        /* RF: not routed */
            } else {
                for (int i = 0; i < N; i++) {
                    const uint16_t *row = K + b * stride_b + h * stride_h + ((int64_t)c * N + i) * stride_s;
                    for (int d = 0; d < D; d++) x[d] = H2F(row[d]);
                    float p[8];
                    router_token_logits(x, D, M, w1, w2, w3, logit_bias, p);
                    int top = 0;
                    for (int k = 1; k < M; k++) if (p[k] > p[top]) top = k;
                    cnt[top] += 1;
                }
                best = 0;
                for (int k = 1; k < M; k++) if (cnt[k] > cnt[best]) best = k;
            }
            expert[u * expert_stride_bh + c] = (uint8_t)best;
            if (votes) for (int k = 0; k < M; k++) votes[(u * expert_stride_bh + c) * M + k] = cnt[k];
        }
        free(x);
    }
    free(w1); free(w2);
    return REF_OK;
}

/* ------------------------------------------------------------------ */
/* Quantiser (Sec. 3.1 only says that a chunk is quantised at the       */
/* bit-width its router chose; the formula is this build's own):        */
/* per token row, per group of G consecutive head-dim elements,         */
/* asymmetric uniform, scale and zero kept as fp16.  Inputs must be     */
/* finite: Inf / NaN have no defined codes.  With k_per_channel the     */
/* keys' groups run along tokens instead (G tokens of one dim), the     */
/* values' groups stay as they are.                                     */
/* ------------------------------------------------------------------ */

/* One group: x[G] fp16 bit patterns in, codes[G] out, *meta = scale | zero<<16. */
void moqae_ref_quantize_group(const uint16_t *x, int G, int bits, uint8_t *codes, uint32_t *meta)
{
    const float qmax = (float)((1 << bits) - 1);
    float mn = H2F(x[0]), mx = H2F(x[0]);
    for (int i = 1; i < G; i++) {
        float v = H2F(x[i]);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    if (mn == 0.0f) mn = 0.0f;                                     /* -0 is stored as +0 */
    if (mx == 0.0f) mx = 0.0f;
    float R   = mx - mn;
    float s32 = R / qmax;
    uint16_t s16 = F2H(s32);
    if (H2F(s16) < s32) s16 = (uint16_t)(s16 + 1);                 /* scale is rounded UP */
    if (s16 == 0) s16 = 0x3C00;                                    /* constant group: scale 1 */
    float s   = H2F(s16);
    float inv = 1.0f / s;
    for (int i = 0; i < G; i++) {
        float t = (H2F(x[i]) - mn) * inv;
        float c = rintf(t);                                        /* ties to even */
        if (c < 0.0f) c = 0.0f;
        if (c > qmax) c = qmax;
        codes[i] = (uint8_t)c;
    }
    *meta = (uint32_t)s16 | ((uint32_t)F2H(mn) << 16);
}

/* Where a code lives.  Codes sit in little-endian 32-bit words; a word
 * carries n = 32/b codes, and the code with in-word index e occupies bits
 * [16*(e%2) + b*(e/2), +b): even e in the low half-word, odd e in the high
 * half-word, so that one mask isolates a pair (e, e+1).
 *
 * K codes: token-major rows.  Row t holds D*b/32 words; in-row word d / n,
 *          in-word index d % n.
 * V codes: dimension-major inside blocks of tokens, cut into tiles of up to
 *          64 slots x 4 words (1 KiB).  With TW = 32/b tokens per word, a slot
 *          holds a slice of TQ = max(TW, 8) consecutive tokens of one
 *          dimension (WD = TQ/TW words) for CPK = 4/WD dimensions that lie 16
 *          apart.  A token block is TB = min(4*TQ, max(N, TQ)) tokens = QD = TB/TQ
 *          slices (QD = 4 for chunks of 64 tokens and more; a shorter chunk is one
 *          block of QD = 1, 2 or 4 slices and a tile has 16*QD slots; a chunk of 8
 *          tokens at 2 bits fills half of its one slice, the rest stays zero); token t
 *          of the chunk sits in block t / TB, slice qd = (t % TB) / TQ, and
 *          inside the slice in word w = (t % TQ) / TW at in-word index
 *          e = t % TW.  Dimension d = 16*ct + j belongs to tile cg = ct / CPK of
 *          its block (D / (16*CPK) tiles per block), slot 16*qd + j, word
 *          n = (ct % CPK) * WD + w of the slot:
 *              word index = ((block * D/(16*CPK) + cg) * 16*QD + 16*qd + j) * 4 + n.
 *          Needs D % 64 == 0 and N % 64 == 0 or N in {8, 16, 32}.            */
static void k_code_pos(int t, int d, int D, int b, uint32_t *word, int *bit)
{
    int n = 32 / b, e = d % n;
    *word = (uint32_t)t * (uint32_t)(D * b / 32) + (uint32_t)(d / n);
    *bit  = 16 * (e % 2) + b * (e / 2);
}
static void v_code_pos(int t, int d, int N, int D, int b, uint32_t *word, int *bit)
{
    int TW = 32 / b, TQ = TW > 8 ? TW : 8, WD = TQ / TW, CPK = 4 / WD;
    int room = N < TQ ? TQ : N;
    int TB = 4 * TQ < room ? 4 * TQ : room, QD = TB / TQ;
    int block = t / TB, qd = (t % TB) / TQ, w = (t % TQ) / TW, e = t % TW;
    int ct = d / 16, j = d % 16, cg = ct / CPK, n = (ct % CPK) * WD + w;
    *word = (uint32_t)(((block * (D / (16 * CPK)) + cg) * (16 * QD) + 16 * qd + j) * 4 + n);
    *bit  = 16 * (e % 2) + b * (e / 2);
}
/* The V layout above exists for quantised experts only when it tiles evenly. */
static int layout_ok(const moqae_ref_cfg *c)
{
    for (int j = 0; j < c->n_experts; j++)
        if (c->expert_bits[j] < 16 && (c->head_dim % 64 || (c->chunk % 64 && c->chunk != 32 && c->chunk != 16 && c->chunk != 8))) return 0;
    return 1;
}

static void put_code(uint8_t *area, uint32_t word, int bit, uint32_t code)
{
    uint32_t w; memcpy(&w, area + 4u * word, 4);                   /* little-endian host */
    w |= code << bit;
    memcpy(area + 4u * word, &w, 4);
}
static uint32_t get_code(const uint8_t *area, uint32_t word, int bit, int b)
{
    uint32_t w; memcpy(&w, area + 4u * word, 4);
    return (w >> bit) & ((1u << b) - 1u);
}

/* Pack one chunk (N rows of K and of V, row stride `ss` elements) into `blk`. */
void moqae_ref_pack_chunk(const moqae_ref_cfg *cfg, int bits,
                          const uint16_t *Kc, const uint16_t *Vc, int64_t ss, uint8_t *blk)
{
    const int N = cfg->chunk, D = cfg->head_dim, G = cfg->group, NG = D / G;
    if (bits == 16) {
        for (int t = 0; t < N; t++) memcpy(blk + (size_t)t * D * 2, Kc + t * ss, (size_t)D * 2);
        blk += (size_t)N * D * 2;
        for (int t = 0; t < N; t++) memcpy(blk + (size_t)t * D * 2, Vc + t * ss, (size_t)D * 2);
        return;
    }
    const size_t code_bytes = (size_t)N * D * bits / 8, meta_bytes = (size_t)N * NG * 4;
    const size_t v_code_bytes = (size_t)v_token_room(N, bits) * D * bits / 8;
    uint8_t *k_codes = blk, *k_meta = k_codes + code_bytes;
    uint8_t *v_codes = k_meta + meta_bytes, *v_meta = v_codes + v_code_bytes;
    memset(blk, 0, code_bytes + v_code_bytes + 2 * meta_bytes);
    uint8_t *codes = malloc((size_t)G);
    /* Keys quantised per channel (the outlier channels of key caches that Sec. 2.2 quotes from KIVI make a group
     * of dims share one huge range; along tokens a channel is homogeneous): a group is G consecutive tokens of one
     * dim, its meta word sits at [token group][dim]; the codes keep their token-major places.                     */
    if (cfg->k_per_channel) {
        uint16_t *col = malloc(sizeof(uint16_t) * (size_t)G);
        for (int tg = 0; tg < N / G; tg++) for (int d = 0; d < D; d++) {
            uint32_t meta, word; int bit;
            for (int i = 0; i < G; i++) col[i] = Kc[(int64_t)(tg * G + i) * ss + d];
            moqae_ref_quantize_group(col, G, bits, codes, &meta);
            memcpy(k_meta + 4u * (size_t)(tg * D + d), &meta, 4);
            for (int i = 0; i < G; i++) {
                k_code_pos(tg * G + i, d, D, bits, &word, &bit);
                put_code(k_codes, word, bit, codes[i]);
            }
        }
        free(col);
    }
    for (int t = 0; t < N; t++) {
        for (int g = 0; g < NG; g++) {
            uint32_t meta, word; int bit;
            if (!cfg->k_per_channel) {
                moqae_ref_quantize_group(Kc + t * ss + g * G, G, bits, codes, &meta);
                memcpy(k_meta + 4u * (size_t)(t * NG + g), &meta, 4);
                for (int i = 0; i < G; i++) {
                    k_code_pos(t, g * G + i, D, bits, &word, &bit);
                    put_code(k_codes, word, bit, codes[i]);
                }
            }
            moqae_ref_quantize_group(Vc + t * ss + g * G, G, bits, codes, &meta);
            memcpy(v_meta + 4u * (size_t)(t * NG + g), &meta, 4);
            for (int i = 0; i < G; i++) {
                v_code_pos(t, g * G + i, N, D, bits, &word, &bit);
                put_code(v_codes, word, bit, codes[i]);
            }
        }
    }
    free(codes);
}

/* Decode one chunk block to binary64: x^ = code * scale + zero, exactly. */
void moqae_ref_decode_chunk(const moqae_ref_cfg *cfg, int bits, const uint8_t *blk,
                            double *Kh, double *Vh)
{
    const int N = cfg->chunk, D = cfg->head_dim, G = cfg->group, NG = D / G;
    if (bits == 16) {
        const uint8_t *kp = blk, *vp = blk + (size_t)N * D * 2;
        for (int i = 0; i < N * D; i++) {
            uint16_t a, b; memcpy(&a, kp + 2 * (size_t)i, 2); memcpy(&b, vp + 2 * (size_t)i, 2);
            Kh[i] = (double)H2F(a); Vh[i] = (double)H2F(b);
        }
        return;
    }
    const size_t code_bytes = (size_t)N * D * bits / 8, meta_bytes = (size_t)N * NG * 4;
    const size_t v_code_bytes = (size_t)v_token_room(N, bits) * D * bits / 8;
    const uint8_t *k_codes = blk, *k_meta = k_codes + code_bytes;
    const uint8_t *v_codes = k_meta + meta_bytes, *v_meta = v_codes + v_code_bytes;
    for (int t = 0; t < N; t++) for (int d = 0; d < D; d++) {
        uint32_t mk, mv, word; int bit;
        memcpy(&mk, k_meta + 4u * (size_t)(cfg->k_per_channel ? (t / G) * D + d : t * NG + d / G), 4);
        memcpy(&mv, v_meta + 4u * (size_t)(t * NG + d / G), 4);
        k_code_pos(t, d, D, bits, &word, &bit);
        Kh[t * D + d] = (double)get_code(k_codes, word, bit, bits) * (double)H2F((uint16_t)(mk & 0xffffu))
                      + (double)H2F((uint16_t)(mk >> 16));
        v_code_pos(t, d, N, D, bits, &word, &bit);
        Vh[t * D + d] = (double)get_code(v_codes, word, bit, bits) * (double)H2F((uint16_t)(mv & 0xffffu))
                      + (double)H2F((uint16_t)(mv >> 16));
    }
}

/* Quantise-and-pack chunks [chunk_begin, chunk_end) of every (b, h).
 * Blocks are laid in (b, h, c) order from *arena_used rounded up to 256 bytes
 * (each block start is a multiple of 256 bytes); chunk_off receives each
 * block's byte offset and *arena_used the new end.
 * *status must be 0 on entry, else the call does nothing.  If the blocks do
 * not fit below arena_capacity (REF_E_ARENA) or an expert index is out of
 * range (REF_E_INVAL), *status is set and nothing else is written.        */
int moqae_quantize_pack_ref(const moqae_ref_cfg *cfg,
                            const uint16_t *K, const uint16_t *V,
                            int64_t stride_b, int64_t stride_h, int64_t stride_s,
                            int32_t chunk_begin, int32_t chunk_end,
                            const uint8_t *expert, int64_t expert_stride_bh,
                            uint8_t *arena, uint64_t arena_capacity, uint64_t *arena_used,
                            uint64_t *chunk_off, int64_t off_stride_bh,
                            int32_t *status)
{
    if (!cfg_ok(cfg) || !layout_ok(cfg) || !K || !V || !expert || !arena || !arena_used || !chunk_off || !status) return REF_E_INVAL;
    if (chunk_begin < 0 || chunk_end < chunk_begin) return REF_E_INVAL;
    if (expert_stride_bh < chunk_end || off_stride_bh < chunk_end) return REF_E_INVAL;
    if (*status != 0) return REF_OK;
    const int N = cfg->chunk;
    const int64_t units = (int64_t)cfg->batch * cfg->n_kv_heads;
    const int64_t nc = chunk_end - chunk_begin;

    /* pass 0: does everything fit? */
    uint64_t pos = round_up_256(*arena_used);
    for (int64_t u = 0; u < units; u++) for (int c = chunk_begin; c < chunk_end; c++) {
        int e = expert[u * expert_stride_bh + c];
        if (e >= cfg->n_experts) { *status = REF_E_INVAL; return REF_OK; }
        pos += round_up_256(moqae_ref_chunk_block_bytes(cfg, cfg->expert_bits[e]));
    }
    if (pos > arena_capacity) { *status = REF_E_ARENA; return REF_OK; }

    /* pass 1: the offset plan, in (b, h, c) order */
    pos = round_up_256(*arena_used);
    for (int64_t u = 0; u < units; u++) for (int c = chunk_begin; c < chunk_end; c++) {
        int e = expert[u * expert_stride_bh + c];
        chunk_off[u * off_stride_bh + c] = pos;
        pos += round_up_256(moqae_ref_chunk_block_bytes(cfg, cfg->expert_bits[e]));
    }
    *arena_used = pos;

    /* pass 2: fill the blocks */
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < units * nc; i++) {
        const int64_t u = i / nc; const int c = chunk_begin + (int)(i % nc);
        const int64_t b = u / cfg->n_kv_heads, h = u % cfg->n_kv_heads;
        const int bits = cfg->expert_bits[expert[u * expert_stride_bh + c]];
        const int64_t base = b * stride_b + h * stride_h + (int64_t)c * N * stride_s;
        moqae_ref_pack_chunk(cfg, bits, K + base, V + base, stride_s, arena + chunk_off[u * off_stride_bh + c]);
    }
    return REF_OK;
}

/* ------------------------------------------------------------------ */
/* Paged store: one pool of fixed-size pages per expert instead of the  */
/* ordered arena, so that a chunk can be routed (Eq. (1)-(2), Sec. 3.2) */
/* and quantised in one pass -- its place no longer depends on the      */
/* decisions of the chunks before it -- and so that chunks can be given */
/* back (a finished sequence, a sliding window).  Not in the paper: it  */
/* stores the same blocks as above, only somewhere else.                */
/*                                                                      */
/* Pool j serves expert j: n_pages[j] pages of                          */
/* round_up_256(chunk_block_bytes(B_j)) bytes, pool after pool in the   */
/* arena.  State (uint32 words): head[8], tail[8], 16 reserved words,    */
/* then the free rings of the pools one after another (n_pages[j]       */
/* entries each, the first at word 32).  The free pages                 */
/* of pool j are ring[head % n] .. ring[(tail-1) % n]; a page is taken  */
/* at head, given back at tail.                                         */
/* ------------------------------------------------------------------ */
typedef struct { int32_t n_pages[8]; } moqae_ref_pool_cfg;

static int pool_ok(const moqae_ref_cfg *c, const moqae_ref_pool_cfg *pc)
{
    if (!pc) return 0;
    for (int j = 0; j < c->n_experts; j++) if (pc->n_pages[j] < 0) return 0;
    return 1;
}
uint64_t moqae_ref_pool_page_bytes(const moqae_ref_cfg *c, int32_t j)
{
    return round_up_256(moqae_ref_chunk_block_bytes(c, c->expert_bits[j]));
}
uint64_t moqae_ref_pool_base(const moqae_ref_cfg *c, const moqae_ref_pool_cfg *pc, int32_t j)
{
    uint64_t off = 0;
    for (int i = 0; i < j; i++) off += (uint64_t)pc->n_pages[i] * moqae_ref_pool_page_bytes(c, i);
    return off;
}
uint64_t moqae_ref_pool_arena_bytes(const moqae_ref_cfg *c, const moqae_ref_pool_cfg *pc)
{
    return moqae_ref_pool_base(c, pc, c->n_experts);
}
static uint32_t ring_start(const moqae_ref_cfg *c, const moqae_ref_pool_cfg *pc, int j)
{
    uint32_t w = 32;
    (void)c;
    for (int i = 0; i < j; i++) w += (uint32_t)pc->n_pages[i];
    return w;
}
uint64_t moqae_ref_pool_state_bytes(const moqae_ref_cfg *c, const moqae_ref_pool_cfg *pc)
{
    return 4u * (uint64_t)ring_start(c, pc, c->n_experts);
}
int moqae_pool_init_ref(const moqae_ref_cfg *cfg, const moqae_ref_pool_cfg *pc, uint32_t *state)
{
    if (!cfg_ok(cfg) || !pool_ok(cfg, pc) || !state) return REF_E_INVAL;
    for (int j = 0; j < 8; j++) { state[j] = 0; state[8 + j] = j < cfg->n_experts ? (uint32_t)pc->n_pages[j] : 0u; }
    for (int j = 16; j < 32; j++) state[j] = 0;
    for (int j = 0; j < cfg->n_experts; j++)
        for (int i = 0; i < pc->n_pages[j]; i++) state[ring_start(cfg, pc, j) + (uint32_t)i] = (uint32_t)i;
    return REF_OK;
}

/* Route (W1 != NULL; else `expert` is an input: the decisions of a routing-sharing leader, Sec. 3.4), take a page of
 * the routed expert's pool and pack, for chunks [chunk_begin, chunk_end) of every (b, h), in (b, h, c) order.
 * chunk_off receives the page's byte offset in the arena.  A chunk whose pool is empty gets offset ~0, is not
 * packed, and *status becomes REF_E_ARENA; an expert index >= M (given decisions) likewise with REF_E_INVAL.
 * *status != 0 on entry: nothing is done.                                                                    */
int moqae_route_pack_paged_ref(const moqae_ref_cfg *cfg, const moqae_ref_pool_cfg *pc,
                               const uint16_t *K, const uint16_t *V,
                               int64_t stride_b, int64_t stride_h, int64_t stride_s,
                               int32_t chunk_begin, int32_t chunk_end,
                               const uint16_t *W1, const uint16_t *W2, const uint16_t *W3, const float *logit_bias,
                               uint8_t *expert, int64_t expert_stride_bh, int32_t *votes,
                               uint8_t *arena, uint32_t *state,
                               uint64_t *chunk_off, int64_t off_stride_bh, int32_t *status)
{
    if (!cfg_ok(cfg) || !layout_ok(cfg) || !pool_ok(cfg, pc) || !K || !V || !expert || !arena || !state || !chunk_off || !status)
        return REF_E_INVAL;
    if (chunk_begin < 0 || chunk_end < chunk_begin || expert_stride_bh < chunk_end || off_stride_bh < chunk_end) return REF_E_INVAL;
    if (W1 && (!W2 || !W3)) return REF_E_INVAL;
    if (*status != 0) return REF_OK;
    if (W1) {
        int rc = moqae_route_chunks_ref(cfg, K, stride_b, stride_h, stride_s, chunk_begin, chunk_end, W1, W2, W3, logit_bias,
                                        expert, expert_stride_bh, votes);
        if (rc != REF_OK) return rc;
    }
    const int N = cfg->chunk;
    const int64_t units = (int64_t)cfg->batch * cfg->n_kv_heads;
    for (int64_t u = 0; u < units; u++) for (int c = chunk_begin; c < chunk_end; c++) {
        const int64_t b = u / cfg->n_kv_heads, h = u % cfg->n_kv_heads;
        const int e = expert[u * expert_stride_bh + c];
        chunk_off[u * off_stride_bh + c] = ~(uint64_t)0;
        if (e >= cfg->n_experts) { *status = REF_E_INVAL; continue; }
        uint32_t *head = &state[e], *tail = &state[8 + e];
        if (*head == *tail) { if (*status == 0) *status = REF_E_ARENA; continue; }
        const uint32_t page = state[ring_start(cfg, pc, e) + *head % (uint32_t)pc->n_pages[e]];
        *head += 1;
        const uint64_t off = moqae_ref_pool_base(cfg, pc, e) + (uint64_t)page * moqae_ref_pool_page_bytes(cfg, e);
        chunk_off[u * off_stride_bh + c] = off;
        const int64_t base = b * stride_b + h * stride_h + (int64_t)c * N * stride_s;
        moqae_ref_pack_chunk(cfg, cfg->expert_bits[e], K + base, V + base, stride_s, arena + off);
    }
    return REF_OK;
}

/* Gives the pages of chunks [chunk_begin, chunk_end) of rows [row_begin, row_end) back to their pools, in (row, c)
 * order, and sets their offsets to ~0.  Chunks without a page (offset ~0) are skipped.                          */
int moqae_pool_release_ref(const moqae_ref_cfg *cfg, const moqae_ref_pool_cfg *pc,
                           const uint8_t *expert, int64_t expert_stride_bh,
                           uint64_t *chunk_off, int64_t off_stride_bh,
                           int32_t row_begin, int32_t row_end, int32_t chunk_begin, int32_t chunk_end, uint32_t *state)
{
    if (!cfg_ok(cfg) || !pool_ok(cfg, pc) || !expert || !chunk_off || !state) return REF_E_INVAL;
    if (row_begin < 0 || row_end < row_begin || row_end > cfg->batch * cfg->n_kv_heads) return REF_E_INVAL;
    if (chunk_begin < 0 || chunk_end < chunk_begin || expert_stride_bh < chunk_end || off_stride_bh < chunk_end) return REF_E_INVAL;
    for (int64_t u = row_begin; u < row_end; u++) for (int c = chunk_begin; c < chunk_end; c++) {
        const uint64_t off = chunk_off[u * off_stride_bh + c];
        const int e = expert[u * expert_stride_bh + c];
        if (off == ~(uint64_t)0 || e >= cfg->n_experts) continue;
        const uint32_t page = (uint32_t)((off - moqae_ref_pool_base(cfg, pc, e)) / moqae_ref_pool_page_bytes(cfg, e));
        state[ring_start(cfg, pc, e) + state[8 + e] % (uint32_t)pc->n_pages[e]] = page;
        state[8 + e] += 1;
        chunk_off[u * off_stride_bh + c] = ~(uint64_t)0;
    }
    return REF_OK;
}

/* ------------------------------------------------------------------ */
/* Decode attention: one query per query head, over the whole cache.    */
/* K^, V^ are built explicitly (decoded chunks, then the FP16 residual  */
/* rows), then o = softmax(scale * q K^T) V in binary64.  Query head hq */
/* reads KV head hq / (Hq/Hkv).                                         */
/* ------------------------------------------------------------------ */
int moqae_decode_attn_ref(const moqae_ref_cfg *cfg,
                          const uint16_t *q,
                          const uint8_t *arena, const uint64_t *chunk_off, const uint8_t *expert,
                          int64_t desc_stride_bh, int32_t n_chunks,
                          const uint16_t *K_tail, const uint16_t *V_tail, int32_t n_tail,
                          double softmax_scale,
                          double *out)
{
    if (!cfg_ok(cfg) || !layout_ok(cfg) || !q || !out) return REF_E_INVAL;
    if (n_chunks < 0 || n_tail < 0 || n_tail >= cfg->chunk) return REF_E_INVAL;
    if (n_chunks > 0 && (!arena || !chunk_off || !expert || desc_stride_bh < n_chunks)) return REF_E_INVAL;
    if (n_tail > 0 && (!K_tail || !V_tail)) return REF_E_INVAL;
    if (n_chunks == 0 && n_tail == 0) return REF_E_INVAL;
    const int N = cfg->chunk, D = cfg->head_dim, Hq = cfg->n_q_heads, Hkv = cfg->n_kv_heads;
    const int rep = Hq / Hkv;
    const int64_t S = (int64_t)n_chunks * N + n_tail;
    const int64_t units = (int64_t)cfg->batch * Hkv;
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; u++) {
        const int64_t b = u / Hkv, h = u % Hkv;
        double *Kh = malloc(sizeof(double) * S * D), *Vh = malloc(sizeof(double) * S * D);
        double *sc = malloc(sizeof(double) * S);
        for (int c = 0; c < n_chunks; c++) {
            int e = expert[u * desc_stride_bh + c];
            if (e >= cfg->n_experts) { bad = 1; continue; }
            moqae_ref_decode_chunk(cfg, cfg->expert_bits[e], arena + chunk_off[u * desc_stride_bh + c],
                                   Kh + (int64_t)c * N * D, Vh + (int64_t)c * N * D);
        }
        for (int t = 0; t < n_tail; t++) for (int d = 0; d < D; d++) {
            int64_t src = (u * N + t) * D + d, dst = ((int64_t)n_chunks * N + t) * D + d;
            Kh[dst] = (double)H2F(K_tail[src]); Vh[dst] = (double)H2F(V_tail[src]);
        }
        for (int r = 0; r < rep; r++) {
            const int64_t hq = h * rep + r;
            const uint16_t *qv = q + (b * Hq + hq) * D;
            double m = -INFINITY;
            for (int64_t t = 0; t < S; t++) {
                double acc = 0.0;
                for (int d = 0; d < D; d++) acc += (double)H2F(qv[d]) * Kh[t * D + d];
                sc[t] = softmax_scale * acc;
                if (sc[t] > m) m = sc[t];
            }
            double l = 0.0;
            for (int64_t t = 0; t < S; t++) { sc[t] = exp(sc[t] - m); l += sc[t]; }
            double *o = out + (b * Hq + hq) * D;
            for (int d = 0; d < D; d++) {
                double acc = 0.0;
                for (int64_t t = 0; t < S; t++) acc += sc[t] * Vh[t * D + d];
                o[d] = acc / l;
            }
        }
        free(Kh); free(Vh); free(sc);
    }
    return bad ? REF_E_INVAL : REF_OK;
}

/* ------------------------------------------------------------------ */
/* Several new tokens per sequence at once (speculative decoding,       */
/* chunked prefill): n_queries queries per head; their own K, V rows    */
/* are the LAST n_queries valid rows of the FP16 residual, and query t  */
/* (0-based) attends to every packed chunk and to the residual rows     */
/* before and including its own: the first n_tail - (n_queries - 1 - t) */
/* rows.  It is n_queries calls of the single-token attention above.    */
/* q, out: [B, n_queries, Hq, D].                                       */
/* ------------------------------------------------------------------ */
int moqae_decode_attn_multi_ref(const moqae_ref_cfg *cfg,
                                const uint16_t *q, int32_t n_queries,
                                const uint8_t *arena, const uint64_t *chunk_off, const uint8_t *expert,
                                int64_t desc_stride_bh, int32_t n_chunks,
                                const uint16_t *K_tail, const uint16_t *V_tail, int32_t n_tail,
                                double softmax_scale,
                                double *out)
{
    if (!cfg_ok(cfg) || !q || !out || n_queries < 1 || n_tail < n_queries) return REF_E_INVAL;
    const int D = cfg->head_dim, Hq = cfg->n_q_heads, B = cfg->batch;
    uint16_t *q1 = malloc(sizeof(uint16_t) * (size_t)B * Hq * D);
    double *o1 = malloc(sizeof(double) * (size_t)B * Hq * D);
    int rc = REF_OK;
    for (int t = 0; t < n_queries && rc == REF_OK; t++) {
        for (int b = 0; b < B; b++)
            memcpy(q1 + (size_t)b * Hq * D, q + ((size_t)b * n_queries + t) * Hq * D, sizeof(uint16_t) * (size_t)Hq * D);
        rc = moqae_decode_attn_ref(cfg, q1, arena, chunk_off, expert, desc_stride_bh, n_chunks, K_tail, V_tail,
                                   n_tail - (n_queries - 1 - t), softmax_scale, o1);
        for (int b = 0; b < B; b++)
            memcpy(out + ((size_t)b * n_queries + t) * Hq * D, o1 + (size_t)b * Hq * D, sizeof(double) * (size_t)Hq * D);
    }
    free(q1); free(o1);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Router fine-tuning loss (Sec. 3.3, Eq. (3)-(5)) and its gradient.    */
/*   L_model = (1/T) sum_i [argmax_k p^i_k = j] p^i_j L_nll / B_j       */
/*   L_mem   = (1/T) sum_i [argmax_k p^i_k = j] 16 p^i_j / B_j          */
/*   L       = lambda L_model + (1 - lambda) L_mem                      */
/* Readings: i runs over the router's outputs, one per cached key row   */
/* (Eq. (1) gives one row of P per token), T of them in all; p^i is the */
/* softmax of the token's logits (the text calls them probabilities,    */
/* Eq. (1) has no softmax); the indicator picks the token's own top-1   */
/* expert j, so a token contributes p^i_j times the penalty of j; L_nll */
/* is the frozen model's loss of the token's sequence (an input here:   */
/* one value per sequence); the two penalty vectors are inputs          */
/* (1/B_j and 16/B_j as printed; the text under Eq. (4) describes the   */
/* second as inverted, which B_j/16 would be).  The top-1 index is      */
/* taken from the router's binary32 logits exactly as in routing; given */
/* it, loss and gradient are evaluated in binary64.                     */
/* Gradient: dL/dlogit_k = w_j p_j (delta_jk - p_k) / T with            */
/* w_j = lambda L_nll pen_model_j + (1-lambda) pen_mem_j, then back     */
/* through logit = h W3 + bias, h = SiLU(z), z = (x W1) * (x W2).       */
/* ------------------------------------------------------------------ */
int moqae_router_loss_grad_ref(const moqae_ref_cfg *cfg,
                               const uint16_t *K, int64_t stride_b, int64_t stride_h, int64_t stride_s,
                               int32_t token_begin, int32_t token_end,
                               const uint16_t *W1, const uint16_t *W2, const uint16_t *W3, const float *logit_bias,
                               const float *nll, const float *pen_model, const float *pen_mem, double lambda,
                               double *loss3, double *dW1, double *dW2, double *dW3, double *dbias)
{
    if (!cfg_ok(cfg) || !K || !W1 || !W2 || !W3 || !nll || !pen_model || !pen_mem || !loss3 || !dW1 || !dW2 || !dW3) return REF_E_INVAL;
    if (token_begin < 0 || token_end <= token_begin) return REF_E_INVAL;
    const int D = cfg->head_dim, M = cfg->n_experts;
    float *w1 = malloc(sizeof(float) * D * M), *w2 = malloc(sizeof(float) * D * M), w3[64];
    float *x = malloc(sizeof(float) * D);
    for (int i = 0; i < D * M; i++) { w1[i] = H2F(W1[i]); w2[i] = H2F(W2[i]); }
    for (int i = 0; i < M * M; i++) w3[i] = H2F(W3[i]);
    const double T = (double)cfg->batch * cfg->n_kv_heads * (double)(token_end - token_begin);
    loss3[0] = loss3[1] = loss3[2] = 0.0;
    for (int i = 0; i < D * M; i++) { dW1[i] = 0.0; dW2[i] = 0.0; }
    for (int i = 0; i < M * M; i++) dW3[i] = 0.0;
    if (dbias) for (int k = 0; k < M; k++) dbias[k] = 0.0;
    for (int64_t b = 0; b < cfg->batch; b++) for (int64_t h = 0; h < cfg->n_kv_heads; h++)
    for (int64_t t = token_begin; t < token_end; t++) {
        const uint16_t *row = K + b * stride_b + h * stride_h + t * stride_s;
        for (int d = 0; d < D; d++) x[d] = H2F(row[d]);
        float p32[8];
        router_token_logits(x, D, M, w1, w2, w3, logit_bias, p32);     /* the routing arithmetic decides the expert */
        int j = 0;
        for (int k = 1; k < M; k++) if (p32[k] > p32[j]) j = k;
        /* forward in binary64 */
        double a[8], bb[8], z[8], sg[8], hh[8], lg[8], p[8];
        for (int m = 0; m < M; m++) {
            a[m] = 0.0; bb[m] = 0.0;
            for (int d = 0; d < D; d++) { a[m] += (double)x[d] * w1[d * M + m]; bb[m] += (double)x[d] * w2[d * M + m]; }
            z[m] = a[m] * bb[m]; sg[m] = 1.0 / (1.0 + exp(-z[m])); hh[m] = z[m] * sg[m];
        }
        double mx = -INFINITY, den = 0.0;
        for (int k = 0; k < M; k++) {
            lg[k] = logit_bias ? (double)logit_bias[k] : 0.0;
            for (int m = 0; m < M; m++) lg[k] += hh[m] * w3[m * M + k];
            if (lg[k] > mx) mx = lg[k];
        }
        for (int k = 0; k < M; k++) { p[k] = exp(lg[k] - mx); den += p[k]; }
        for (int k = 0; k < M; k++) p[k] /= den;
        const double lm = p[j] * (double)nll[b] * (double)pen_model[j], le = p[j] * (double)pen_mem[j];
        loss3[1] += lm / T; loss3[2] += le / T;
        /* backward */
        const double w = lambda * (double)nll[b] * (double)pen_model[j] + (1.0 - lambda) * (double)pen_mem[j];
        double dl[8], dh[8];
        for (int k = 0; k < M; k++) dl[k] = w * p[j] * ((k == j ? 1.0 : 0.0) - p[k]) / T;
        for (int m = 0; m < M; m++) {
            dh[m] = 0.0;
            for (int k = 0; k < M; k++) { dh[m] += dl[k] * w3[m * M + k]; dW3[m * M + k] += hh[m] * dl[k]; }
        }
        if (dbias) for (int k = 0; k < M; k++) dbias[k] += dl[k];
        for (int m = 0; m < M; m++) {
            const double dz = dh[m] * (sg[m] * (1.0 + z[m] * (1.0 - sg[m])));    /* d SiLU(z) / dz */
            const double da = dz * bb[m], db = dz * a[m];
            for (int d = 0; d < D; d++) { dW1[d * M + m] += (double)x[d] * da; dW2[d * M + m] += (double)x[d] * db; }
        }
    }
    loss3[0] = lambda * loss3[1] + (1.0 - lambda) * loss3[2];
    free(w1); free(w2); free(x);
    return REF_OK;
}

int moqae_ref_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
