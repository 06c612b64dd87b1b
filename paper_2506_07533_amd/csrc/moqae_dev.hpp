// Device-side helpers shared by the three kernels of libmoqae (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moqae {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int kD = 128;          // head_dim (the only one supported)
constexpr int kWave = 64;

__device__ __forceinline__ float half_bits_to_float(uint32_t h16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h16);
}
__device__ __forceinline__ uint32_t float_to_half_bits(float f) {      // round-to-nearest-even
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}
__device__ __forceinline__ half2_t as_half2(uint32_t w) { return __builtin_bit_cast(half2_t, w); }

// D(f32) = a.lo*b.lo + a.hi*b.hi + c  (v_dot2_f32_f16; fp16 subnormal inputs are kept)
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2(as_half2(a), as_half2(b), c, false);
}

// ---- DPP cross-lane moves (all lanes active) -------------------------------------------
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_f(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
        __builtin_bit_cast(int, x), __builtin_bit_cast(int, x), CTRL, ROW_MASK, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, 0xF, 0xF, false);
}
constexpr int DPP_XOR1 = 0xB1;           // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;           // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;   // lane i <-> 7-i inside 8 lanes
constexpr int DPP_MIRROR = 0x140;        // lane i <-> 15-i inside a row of 16
constexpr int DPP_BCAST15 = 0x142;       // lane 15 of a row -> the next row
constexpr int DPP_BCAST31 = 0x143;       // lane 31 -> rows 2, 3

// Cross-lane reductions with the lane permutation folded into the arithmetic instruction (one vector
// instruction per step).  Written as instructions because the compiler keeps the permutation as a move of
// its own and re-canonicalises its result (four instructions per step).  The compiler does not see what
// an asm statement executes and inserts no wait states for it, so every step brings its own: a DPP
// operand must not be read within two wait states of an ordinary vector instruction that wrote it, nor
// within three of a dot-product instruction (v_dot2_f32_f16 feeds group_sum directly); the first step
// therefore waits three, the later ones (whose producer is the previous step) two, and a last s_nop
// covers whatever DPP instruction may follow.  The input must not be the direct result of a matrix-core
// instruction (their results need far longer).  All lanes must be active.
#define MOQAE_DPP_FIRST(OP, CTRL) asm("s_nop 2\n\t" OP "_dpp %0, %0, %0 " CTRL : "+v"(x))
#define MOQAE_DPP_STEP(OP, CTRL) asm("s_nop 1\n\t" OP "_dpp %0, %0, %0 " CTRL : "+v"(x))
#define MOQAE_DPP_END() asm("s_nop 1" : "+v"(x))
#define MOQAE_DPP_FULL " row_mask:0xf bank_mask:0xf"

// Sum over aligned groups of LANES consecutive lanes (2, 4, 8 or 16); every lane gets the sum.
template <int LANES>
__device__ __forceinline__ float group_sum(float x) {
    if constexpr (LANES >= 2)  MOQAE_DPP_FIRST("v_add_f32", "quad_perm:[1,0,3,2]" MOQAE_DPP_FULL);
    if constexpr (LANES >= 4)  MOQAE_DPP_STEP("v_add_f32", "quad_perm:[2,3,0,1]" MOQAE_DPP_FULL);
    if constexpr (LANES >= 8)  MOQAE_DPP_STEP("v_add_f32", "row_half_mirror" MOQAE_DPP_FULL);
    if constexpr (LANES >= 16) MOQAE_DPP_STEP("v_add_f32", "row_mirror" MOQAE_DPP_FULL);
    MOQAE_DPP_END();
    return x;
}
template <int LANES>
__device__ __forceinline__ float group_min(float x) {
    if constexpr (LANES >= 2)  MOQAE_DPP_FIRST("v_min_f32", "quad_perm:[1,0,3,2]" MOQAE_DPP_FULL);
    if constexpr (LANES >= 4)  MOQAE_DPP_STEP("v_min_f32", "quad_perm:[2,3,0,1]" MOQAE_DPP_FULL);
    if constexpr (LANES >= 8)  MOQAE_DPP_STEP("v_min_f32", "row_half_mirror" MOQAE_DPP_FULL);
    if constexpr (LANES >= 16) MOQAE_DPP_STEP("v_min_f32", "row_mirror" MOQAE_DPP_FULL);
    MOQAE_DPP_END();
    return x;
}
template <int LANES>
__device__ __forceinline__ float group_max(float x) {
    if constexpr (LANES >= 2)  MOQAE_DPP_FIRST("v_max_f32", "quad_perm:[1,0,3,2]" MOQAE_DPP_FULL);
    if constexpr (LANES >= 4)  MOQAE_DPP_STEP("v_max_f32", "quad_perm:[2,3,0,1]" MOQAE_DPP_FULL);
    if constexpr (LANES >= 8)  MOQAE_DPP_STEP("v_max_f32", "row_half_mirror" MOQAE_DPP_FULL);
    if constexpr (LANES >= 16) MOQAE_DPP_STEP("v_max_f32", "row_mirror" MOQAE_DPP_FULL);
    MOQAE_DPP_END();
    return x;
}
// Maximum over the whole wavefront, returned wave-uniform.  After the rows: lane 15 of rows 0 and 2 is
// folded into rows 1 and 3 (the other rows keep their value), then lane 31 into rows 2 and 3; lane 63
// holds the maximum of all.
__device__ __forceinline__ float wave_max(float x) {
    MOQAE_DPP_FIRST("v_max_f32", "quad_perm:[1,0,3,2]" MOQAE_DPP_FULL);
    MOQAE_DPP_STEP("v_max_f32", "quad_perm:[2,3,0,1]" MOQAE_DPP_FULL);
    MOQAE_DPP_STEP("v_max_f32", "row_half_mirror" MOQAE_DPP_FULL);
    MOQAE_DPP_STEP("v_max_f32", "row_mirror" MOQAE_DPP_FULL);
    MOQAE_DPP_STEP("v_max_f32", "row_bcast:15 row_mask:0xa bank_mask:0xf");
    MOQAE_DPP_STEP("v_max_f32", "row_bcast:31 row_mask:0xc bank_mask:0xf");
    MOQAE_DPP_END();
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Tokens the V code area of a chunk has room for: N, but at least one slice of the V layout (max(32/b, 8) tokens):
// 8 tokens at 2 bits take a slice of 16 whose upper half holds zero codes.
__host__ __device__ inline int v_token_room(int N, int b) {
    const int TQ = 32 / b > 8 ? 32 / b : 8;
    return N < TQ ? TQ : N;
}
// Bytes of one chunk block (K and V) at bit-width b.
__host__ __device__ inline uint64_t block_bytes(int N, int G, int b) {
    return b == 16 ? (uint64_t)N * kD * 4u
                   : (uint64_t)(N + v_token_room(N, b)) * kD * (uint64_t)b / 8u + 2u * (uint64_t)N * (kD / G) * 4u;
}

}  // namespace moqae
