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

// 128-bit store with agent scope (the sc1 cache-policy bit): the data is written through to memory at
// once and the line stays valid in L2.  HIP has no builtin for a scoped 128-bit store.  `base` must be
// wave-uniform (it travels in scalar registers), `byte_off` is the lane's offset from it.  The
// instruction reads its operands when it issues, so the registers are free right after it.
// (One dword with the same scope: for the odd words beside such stores -- ordinary stores into cache
// lines that also receive agent-scope stores are very slow.)
__device__ __forceinline__ void store_u32_agent(const void* base, uint32_t byte_off, uint32_t w) {
    asm volatile("global_store_dword %0, %1, %2 sc1" ::"v"(byte_off), "v"(w), "s"(base) : "memory");
}
__device__ __forceinline__ void store_v4u_agent(const void* base, uint32_t byte_off, v4u w) {
    asm volatile("global_store_dwordx4 %0, %1, %2 sc1" ::"v"(byte_off), "v"(w), "s"(base) : "memory");
}

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
// bumped by the Weyl constants between rounds.  NOT: return the complement of the four output words
// (the rounding below consumes 65535 - h); two of the four complements ride along in the last round's
// three-input xor through a complemented key, which is scalar work.
template <bool NOT = false>
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&o)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * (uint64_t)c2;
        const bool flip = NOT && r == 9;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, flip ? ~k0 : k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, flip ? ~k1 : k1);
        c1 = flip ? ~(uint32_t)p1 : (uint32_t)p1;
        c3 = flip ? ~(uint32_t)p0 : (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    o[0] = c0; o[1] = c1; o[2] = c2; o[3] = c3;
}

// Stochastic rounding of one element in 16.16 fixed point.
//
// The code is floor(u) + [(h + 1/2) / 65536 < frac(u)], u = clamp(fma(x, a, L/2), 0, L).  For an integer
// h the comparison says h < T with T = ceil(frac(u) * 65536 - 1/2), the number of the 65536 uniforms
// that round up.  floor(u) * 65536 + T is ceil(u * 65536 - 1/2) =: F, so
//     code = (F + 65535 - h) >> 16
// (the low halves add up to T + 65535 - h, which carries exactly when h < T).  u * 65536 comes out of
// the same fma with both constants scaled by 2^16 -- a power of two moves through the rounding of the
// fma unchanged; where u itself is a denormal both forms give code 0 -- and F is one conversion:
// v_cvt_rpi_i32_f32 returns floor(s + 1/2) exactly, also for |s| >= 2^23, and floor(-v + 1/2) = -F.
// Five vector operations per element (fma, clamp, convert, subtract, shift) where the floating-point
// comparison took eight.
struct FixedGrid {
    float half16;   // (L/2) * 65536
    float top16;    // L * 65536
};
__device__ __forceinline__ FixedGrid fixed_grid(uint32_t bits) {
    const float Lf = (float)((1u << bits) - 1u);
    return FixedGrid{0.5f * Lf * 65536.0f, Lf * 65536.0f};   // exact: L <= 255
}
// a16 = fl((L/2)/s) * 65536; returns -F
__device__ __forceinline__ int neg_fixed_position(float x, float a16, const FixedGrid& g) {
    float v = __builtin_fmaf(x, a16, g.half16);
    v = __builtin_amdgcn_fmed3f(v, 0.0f, g.top16);
    int r;
    asm("v_cvt_rpi_i32_f32_e64 %0, -%1" : "=v"(r) : "v"(v));
    return r;
}
// nh16 = 65535 - h, the complemented 16-bit uniform.  Returns (code << 16) | (16 bits of no interest).
__device__ __forceinline__ uint32_t round_code_hi(float x, float a16, const FixedGrid& g, uint32_t nh16) {
    return nh16 - (uint32_t)neg_fixed_position(x, a16, g);
}

// The four codes of a quad, each in the upper half-word of its register, as one value of 4 * bits bits
// (code 0 lowest).  The shifts and the first or read the upper half-word directly (SDWA operand
// selection), so no separate >> 16 is issued: five operations per quad.  s1, s2, s3 = bits, 2 * bits,
// 3 * bits.
__device__ __forceinline__ uint32_t pack_quad_hi(uint32_t t0, uint32_t t1, uint32_t t2, uint32_t t3,
                                                 uint32_t s1, uint32_t s2, uint32_t s3) {
    uint32_t v1, v2, v3, v0;
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1" : "=v"(v1) : "s"(s1), "v"(t1));
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1" : "=v"(v2) : "s"(s2), "v"(t2));
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1" : "=v"(v3) : "s"(s3), "v"(t3));
    asm("v_or_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1 src1_sel:DWORD" : "=v"(v0) : "v"(t0), "v"(v1));
    return v0 | v2 | v3;
}

}  // namespace encode
}  // namespace mqg
