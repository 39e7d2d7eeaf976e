// Pieces of the quantizer (steps a2, a3 of the hot path) shared by the kernels that write packed
// code streams: lane-exchange helpers, Philox4x32-10, and the stochastic rounding of one element.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mqg {
namespace encode {

constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;

constexpr int kDppQuadSwap1 = 0xB1;       // quad_perm [1,0,3,2]: lane ^ 1
constexpr int kDppQuadSwap2 = 0x4E;       // quad_perm [2,3,0,1]: lane ^ 2
constexpr int kDppRowHalfMirror = 0x141;  // lane i <-> 7 - i inside each group of 8
constexpr int kDppRowMirror = 0x140;      // lane i <-> 15 - i inside each row of 16

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
// the same 128-bit vectors at 4-byte alignment: global memory takes multi-dword accesses at any dword
// address, so a tensor that starts off a 16-byte boundary is still read and written 128 bits at a time
typedef v4f v4f_a4 __attribute__((aligned(4)));
typedef v4u v4u_a4 __attribute__((aligned(4)));

// DPP reads of a switched-off lane return 0: call these with every lane of the wave active.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __builtin_bit_cast(float, dpp_u32<CTRL>(__builtin_bit_cast(uint32_t, v)));
}

// lane ^ 16 and lane ^ 32 exchanges on the LDS pipe (no vector-ALU issue, no LDS memory)
constexpr int kSwizzleXor16 = 0x401F;     // bit-mode swizzle: and 0x1F, or 0, xor 0x10
__device__ __forceinline__ float swizzle_xor16_f32(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), kSwizzleXor16));
}
__device__ __forceinline__ float bpermute_xor32_f32(float v, uint32_t lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((int)((lane ^ 32u) << 2), __builtin_bit_cast(int, v)));
}

// Cross-lane max / min on unsigned integers.  Non-negative floats order like their bit patterns, and
// any float orders like its order-preserving key (order_key below), so the reductions run on integers:
// no NaN canonicalisation is inserted, and the DPP operand folds into the max / min instruction.
// Call with every lane of the wave active.
__device__ __forceinline__ uint32_t cell_max_u32(uint32_t m) {   // over each group of 8 lanes
    m = max(m, dpp_u32<kDppQuadSwap1>(m));
    m = max(m, dpp_u32<kDppQuadSwap2>(m));
    return max(m, dpp_u32<kDppRowHalfMirror>(m));
}
__device__ __forceinline__ uint32_t cell_min_u32(uint32_t m) {
    m = min(m, dpp_u32<kDppQuadSwap1>(m));
    m = min(m, dpp_u32<kDppQuadSwap2>(m));
    return min(m, dpp_u32<kDppRowHalfMirror>(m));
}
__device__ __forceinline__ uint32_t swizzle_xor16_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, kSwizzleXor16);
}
__device__ __forceinline__ uint32_t bpermute_xor32_u32(uint32_t v, uint32_t lane) {
    return (uint32_t)__builtin_amdgcn_ds_bpermute((int)((lane ^ 32u) << 2), (int)v);
}
// from values already reduced over each 8-lane group to the whole wave: every lane gets the result
__device__ __forceinline__ uint32_t wave_max_from_cells_u32(uint32_t m, uint32_t lane) {
    m = max(m, dpp_u32<kDppRowMirror>(m));
    m = max(m, swizzle_xor16_u32(m));
    return max(m, bpermute_xor32_u32(m, lane));
}
__device__ __forceinline__ uint32_t wave_min_from_cells_u32(uint32_t m, uint32_t lane) {
    m = min(m, dpp_u32<kDppRowMirror>(m));
    m = min(m, swizzle_xor16_u32(m));
    return min(m, bpermute_xor32_u32(m, lane));
}

// fp32 -> uint32 whose unsigned order is the order of the floats, and back
__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t u = __builtin_bit_cast(uint32_t, f);
    return u ^ (uint32_t)(((int)u >> 31) | (int)0x80000000);
}
__device__ __forceinline__ float key_value(uint32_t k) {
    const uint32_t u = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
    return __builtin_bit_cast(float, u);
}

// a ^ b ^ c in one instruction: gfx950's three-input bitwise operation with the parity truth table
// (bit i of 0x96 is the parity of i's three bits).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return (uint32_t)__builtin_amdgcn_bitop3_b32((int)a, (int)b, (int)c, 0x96);
}

// Lanes of one wave exchange data through LDS without a workgroup barrier.  The hardware executes a
// wave's LDS instructions in program order, so what one lane wrote is there for the others as soon as
// the instructions are in that order; this fence keeps the COMPILER from moving memory accesses
// across the exchange point (without it a lane's read may legally be hoisted above another lane's
// write: to the compiler they are unordered accesses of different threads).  Wavefront scope: no
// cache maintenance and no instruction beyond the waits the accesses need anyway.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Philox4x32-10 (Salmon et al., SC'11).  Ten rounds of two 32x32->64 multiplies; the key is
// bumped by the Weyl constants between rounds.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&o)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * (uint64_t)c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    o[0] = c0; o[1] = c1; o[2] = c2; o[3] = c3;
}

// code of one element: floor(u) + [(h + 1/2) / 65536 < frac(u)].
// The comparison is evaluated as  h < frac*65536 - 1/2 : the right-hand side is exact in fp32
// whenever it is non-negative (frac*65536 < 2^16 has an ulp of at most 2^-8), and negative
// otherwise, so both forms decide identically for every integer h in [0, 65535].
__device__ __forceinline__ uint32_t round_code(float x, float ainv, float halfL, float Lf, uint32_t h16) {
    float u = __builtin_fmaf(x, ainv, halfL);
    u = __builtin_amdgcn_fmed3f(u, 0.0f, Lf);
    const float fr = __builtin_amdgcn_fractf(u);
    const float t = __builtin_fmaf(fr, 65536.0f, -0.5f);
    const float hf = (float)h16;
    return (uint32_t)u + ((hf < t) ? 1u : 0u);
}

}  // namespace encode
}  // namespace mqg
