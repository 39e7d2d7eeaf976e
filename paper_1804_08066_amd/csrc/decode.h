// Unpack + de-quantize + accumulate (steps a5, a6 of the hot path), shared by the kernels that read
// packed code streams: the server's aggregate_update and its re-quantizing variant.
//
// A lane owns R quads of 4 consecutive elements; quad q of a tile starts at stream bit 4*bits*q of
// the tile's first word.  Its 4 codes lie inside one 32-bit word when bits divides 32 and spill
// into the next word otherwise -- and that next word is the first word of the next lane's quad.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mqgrad.h"

namespace mqg {
namespace decode {

constexpr int kDppWaveShl1 = 0x130;   // DPP wave_shl:1: lane i reads lane i + 1

// Where the codes of the lane's R quads sit in every worker's stream.  A row of the tile is a whole
// number of words (ROW is a multiple of 8 quads), so the bit offset inside the first word is the same
// for every row; the byte offsets are clamped to the last word of the stream so that quads past the
// end still read valid memory (what they decode is never used).
template <int R>
struct CodeWindows {
    uint32_t byte[R];    // byte offset of the quad's first word from the tile's first word (< 2^32)
    uint32_t sh;         // bit offset of the quad's first code inside that word
    uint64_t tile_word;  // first word of the tile in the stream
};

// ROW: quads per row of the tile (the lanes that load one row); `idx`: this lane's index in a row.
// Row j of the lane is quad j*ROW + idx of the tile that starts at element `tile_base`.
template <int R, int ROW>
__device__ __forceinline__ CodeWindows<R> code_windows(uint64_t n, uint64_t tile_base, uint32_t b, uint32_t idx) {
    static_assert(ROW % 8 == 0, "a row is a whole number of words at every width");
    CodeWindows<R> cw;
    cw.tile_word = (tile_base >> 5) * b;   // tile_base is a multiple of 32
    const uint64_t stream_words = (n >> 5) * b + ((((n & 31u) * b) + 31u) >> 5);
    const uint64_t room = stream_words - cw.tile_word;   // >= 1 whenever tile_base < n
    const uint32_t last_word = room - 1u > 0x3FFFFFFFull ? 0x3FFFFFFFu : (uint32_t)(room - 1u);
    const uint32_t bit = 4u * b * idx;
    const uint32_t word = bit >> 5;
    const uint32_t row_words = (ROW / 8) * b;
    cw.sh = bit & 31u;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t wj = word + j * row_words;
        cw.byte[j] = (wj < last_word ? wj : last_word) * 4u;
    }
    return cw;
}

template <int R, int CH>
struct CodeRegs {
    uint32_t lo[CH][R];
};

// A wave's code words of one row and worker are 32*bits contiguous bytes.  From 4 bits on the loads
// carry the streaming hint like every other read-once access; below that neighbouring waves read the
// rest of the same 128-byte line and a streaming load would fetch it from L2 once per wave, so the loads
// are ordinary ones and the vector L1 serves the neighbours.  Measured at 100 M elements, W = 8, with the
// code words written by the quantizer's agent-scope stores just before: the hint is 6-8 % faster at 5
// and 7 bits, level at 4, 6 and 8, and 7-9 % slower at 2 and 3 bits.
inline __host__ __device__ bool codes_read_once(uint32_t b) { return b >= 4u; }

// Fetch the first code word of each of the lane's quads for workers [w0, min(w0 + CH, W)): one
// aligned dword load per worker and quad, all issued before any is consumed.  Adjacent lanes read
// the same or adjacent words, so a wave's request is one contiguous run of 32*bits bytes.
template <int R, int CH, bool ONCE>
__device__ __forceinline__ void fetch_codes(const uint32_t* const* packed, uint32_t W,
                                            uint32_t w0, const CodeWindows<R>& cw, CodeRegs<R, CH>& c) {
#pragma unroll
    for (int t = 0; t < CH; ++t) {
        if (w0 + t < W) {
            // uniform base + 32-bit lane offset: the address costs no vector operation
            const char* __restrict__ src = (const char*)(packed[w0 + t] + cw.tile_word);
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const uint32_t* q = (const uint32_t*)(src + cw.byte[j]);
                c.lo[t][j] = ONCE ? __builtin_nontemporal_load(q) : *q;
            }
        }
    }
}

// The 4 codes of one quad of one worker, from the quad's first word `lo` and its bit offset `sh`.
template <bool STRADDLE>
__device__ __forceinline__ void extract_quad(uint32_t lo, uint32_t sh, uint32_t b, int (&k)[4]) {
    uint32_t v, o;
    if (STRADDLE) {
        // A quad that spills over its first word continues in the first word of the next lane (that
        // lane's quad starts where this one ends), so the second word comes through a one-lane DPP
        // shift instead of a second load.  A wave's 64 quads are 8*bits whole words, so lane 63
        // never spills and what it reads here is never used.  Must run with all lanes active.
        const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lo, kDppWaveShl1, 0xF, 0xF, false);
        v = __builtin_amdgcn_alignbit(hi, lo, sh);   // ({hi,lo} >> sh)[31:0]
        o = 0u;
    } else {
        v = lo;
        o = sh;
    }
    k[0] = (int)__builtin_amdgcn_ubfe(v, o, b);
    k[1] = (int)__builtin_amdgcn_ubfe(v, o + b, b);
    k[2] = (int)__builtin_amdgcn_ubfe(v, o + 2u * b, b);
    k[3] = (int)__builtin_amdgcn_ubfe(v, o + 3u * b, b);
}

// (float)(2c - L) without extracting c: two vector operations per code, where bit-field extract,
// shift-add and convert take three.
// With the b-bit code at bit P of `y` (P = 1 or 1 + b; the other bits of `y` are arbitrary):
//   1. AND with the field mask, OR with the bits of 1.0f: the code becomes mantissa bits of
//      x = 1 + c * 2^(P - 23)  (P + b <= 23 holds for b <= 8);
//   2. one fma: x * 2^(24 - P) - (2^(24 - P) + L) = 2c - L.  Every quantity is a whole number of
//      units 2^(1 - P) <= 1 and below 2^24 units, so the constants are exact and the fma rounds nothing.
// The constants are uniform; the subtrahends are pinned to vector registers (an fma takes one scalar
// operand) so that no use re-materialises them.
struct Centred {
    uint32_t b;
    uint32_t field[2];    // L << P
    float scale[2];       // 2^(24 - P)
    float minus_c[2];     // -(2^(24 - P) + L)
};
__device__ __forceinline__ Centred centred(uint32_t b) {
    const uint32_t L = (1u << b) - 1u;
    Centred cd;
    cd.b = b;
    cd.field[0] = L << 1;
    cd.field[1] = L << (1u + b);
    uint32_t s0 = 150u << 23, s1 = (150u - b) << 23;   // 2^23, 2^(23 - b)
    uint32_t c0 = 0x80000000u | s0 | L, c1 = 0x80000000u | s1 | (L << b);
    asm volatile("" : "+s"(s0), "+s"(s1));
    asm volatile("" : "+v"(c0), "+v"(c1));
    cd.scale[0] = __builtin_bit_cast(float, s0);
    cd.scale[1] = __builtin_bit_cast(float, s1);
    cd.minus_c[0] = __builtin_bit_cast(float, c0);
    cd.minus_c[1] = __builtin_bit_cast(float, c1);
    return cd;
}
__device__ __forceinline__ float centred_code(uint32_t y, const Centred& cd, int place) {
    const float x = __builtin_bit_cast(float, (y & cd.field[place]) | 0x3F800000u);
    return __builtin_fmaf(x, cd.scale[place], cd.minus_c[place]);
}

// One worker's 4 codes of one quad, de-quantized with step d and accumulated:
// acc <- fma((float)(2c - L), d, acc), the ordered chain of the server's sum.
template <bool STRADDLE>
__device__ __forceinline__ void accumulate_quad(uint32_t lo, uint32_t sh, const Centred& cd, float d, float4& acc) {
    // ya holds codes 0 and 1 of the quad at bits 1 and 1 + b, yb codes 2 and 3 at the same places.
    uint32_t ya, yb;
    if (STRADDLE) {
        const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lo, kDppWaveShl1, 0xF, 0xF, false);
        const uint32_t v = __builtin_amdgcn_alignbit(hi, lo, sh);   // as in extract_quad
        ya = v << 1;
        yb = v >> (2u * cd.b - 1u);
    } else {
        ya = __builtin_amdgcn_alignbit(lo, lo, (sh - 1u) & 31u);    // rotate: bit sh moves to bit 1
        yb = __builtin_amdgcn_alignbit(ya, ya, 2u * cd.b);          // rotate again: at 8 bits code 3 wraps round
    }
    acc.x = __builtin_fmaf(centred_code(ya, cd, 0), d, acc.x);
    acc.y = __builtin_fmaf(centred_code(ya, cd, 1), d, acc.y);
    acc.z = __builtin_fmaf(centred_code(yb, cd, 0), d, acc.z);
    acc.w = __builtin_fmaf(centred_code(yb, cd, 1), d, acc.w);
}

// One-bit codes: (2c - L) is +1 or -1, so the fma of the chain is an exactly rounded add or subtract
// of d.  The code bit is shifted to the sign position and XOR-ed into d with one three-input bitwise
// operation ((a & b) ^ c has the truth table 0x6A for a = 0xF0, b = 0xCC, c = 0xAA); what is
// subtracted is -d for a set bit and +d for a clear one: three vector operations per element
// (the general form takes three and a half), bit-identical results.
__device__ __forceinline__ float minus_signed_step(uint32_t word, uint32_t shl, float d) {
    const uint32_t t = word << shl;   // code bit at bit 31
    const int r = __builtin_amdgcn_bitop3_b32((int)t, (int)0x80000000u, __builtin_bit_cast(int, d), 0x6A);
    return __builtin_bit_cast(float, r);
}
__device__ __forceinline__ void accumulate_quad_onebit(uint32_t lo, uint32_t sh, float d, float4& acc) {
    acc.x = acc.x - minus_signed_step(lo, 31u - sh, d);
    acc.y = acc.y - minus_signed_step(lo, 30u - sh, d);
    acc.z = acc.z - minus_signed_step(lo, 29u - sh, d);
    acc.w = acc.w - minus_signed_step(lo, 28u - sh, d);
}

// Eight-bit codes: a quad is the four bytes of one word, and a byte converts to fp32 in one
// instruction (v_cvt_f32_ubyte0..3); 2c - 255 is then one exact fma, so the chain's fma sees the same
// multiplier as in the general path: three vector operations per element, no shifts per quad.
__device__ __forceinline__ void accumulate_quad_bytes(uint32_t lo, float d, float4& acc) {
    const float k0 = (float)(lo & 0xFFu), k1 = (float)((lo >> 8) & 0xFFu);
    const float k2 = (float)((lo >> 16) & 0xFFu), k3 = (float)(lo >> 24);
    acc.x = __builtin_fmaf(__builtin_fmaf(k0, 2.0f, -255.0f), d, acc.x);
    acc.y = __builtin_fmaf(__builtin_fmaf(k1, 2.0f, -255.0f), d, acc.y);
    acc.z = __builtin_fmaf(__builtin_fmaf(k2, 2.0f, -255.0f), d, acc.z);
    acc.w = __builtin_fmaf(__builtin_fmaf(k3, 2.0f, -255.0f), d, acc.w);
}

// Widths 1 to 4 through a table in LDS.  The multiplier (float)(2c - L) depends on the code alone, so the
// pairs (2 c0 - L, 2 c1 - L) of two adjacent codes are tabulated once per workgroup -- 4^bits entries of
// two floats: 32 bytes to 2 KB -- and a lane fetches the two pairs of its quad with two 64-bit LDS reads
// (the LDS pipe, not the vector ALU); at one bit a whole quad indexes a table of 16 entries of four
// floats.  What is left for the vector ALU is one rotation per quad, the two table offsets and the
// chain's own fma per code.  Results are those of the all-fp32 form bit for bit: the table holds the same
// multiplier, and the chain's fma is the same instruction.  Used where the decode's vector operations
// limit the kernel: the fused update with more than eight workers up to 3 bits, the re-quantizing step
// up to 4 bits (the [min, max] re-encoding kernels did not gain: 164 against 149 us).  Wider codes gain
// nothing either: a pair table for 5 bits (8 KB) helped at some
// bucket sizes and hurt at others, one for 6 bits (32 KB) costs more occupancy than the decode saves.
constexpr uint32_t kLutFloats = 512;   // 4^4 entries of two floats
// Filled by `nthreads` threads (tid = 0 .. nthreads - 1); a barrier must follow.
__device__ __forceinline__ void build_pair_lut(float* lut, uint32_t b, uint32_t tid, uint32_t nthreads = 256u) {
    const int L = (int)((1u << b) - 1u);
    const auto value = [&](uint32_t c) { return (float)(2 * (int)c - L); };
    if (b == 1u) {
        if (tid < 64u) lut[tid] = value(((tid >> 2) >> (tid & 3u)) & 1u);   // entry tid / 4, element tid % 4
    } else {
        for (uint32_t e = tid; e < (1u << (2u * b)); e += nthreads) {
            lut[2u * e] = value(e & (uint32_t)L);
            lut[2u * e + 1u] = value(e >> b);
        }
    }
}
// The table entries of one quad: B = bits (1, 2, 4: the quad lies inside one word; 3: it may spill into
// the next lane's word, which arrives through a one-lane DPP shift -- call with all lanes active).
template <int B>
__device__ __forceinline__ float4 lut_quad(uint32_t lo, uint32_t sh, const float* lut) {
    if (B == 1) {
        const uint32_t r = __builtin_amdgcn_alignbit(lo, lo, (sh - 4u) & 31u);   // rotate: bit sh moves to bit 4
        return *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(lut) + (r & 0xF0u));
    }
    constexpr uint32_t kMask = ((1u << (2 * B)) - 1u) << 3;   // a pair's index times the entry size
    uint32_t oa, ob;
    if (B == 3) {
        const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lo, kDppWaveShl1, 0xF, 0xF, false);
        const uint32_t v = __builtin_amdgcn_alignbit(hi, lo, sh);   // the quad's 12 bits at bit 0
        oa = (v << 3) & kMask;
        ob = (v >> 3) & kMask;
    } else {
        const uint32_t r = __builtin_amdgcn_alignbit(lo, lo, (sh - 3u) & 31u);   // rotate: bit sh moves to bit 3
        oa = r & kMask;
        ob = (r >> (2 * B)) & kMask;
    }
    const float2 ma = *reinterpret_cast<const float2*>(reinterpret_cast<const char*>(lut) + oa);
    const float2 mb = *reinterpret_cast<const float2*>(reinterpret_cast<const char*>(lut) + ob);
    return make_float4(ma.x, ma.y, mb.x, mb.y);
}
template <int B>
__device__ __forceinline__ void accumulate_quad_lut(uint32_t lo, uint32_t sh, const float* lut, float d, float4& acc) {
    const float4 m = lut_quad<B>(lo, sh, lut);
    acc.x = __builtin_fmaf(m.x, d, acc.x);
    acc.y = __builtin_fmaf(m.y, d, acc.y);
    acc.z = __builtin_fmaf(m.z, d, acc.z);
    acc.w = __builtin_fmaf(m.w, d, acc.w);
}

// Dispatch on the width class: WIDTH = 1 or 8 select the three-operation forms above, 0 the general one.
template <bool STRADDLE, int WIDTH>
__device__ __forceinline__ void accumulate_quad_w(uint32_t lo, uint32_t sh, const Centred& cd, float d, float4& acc) {
    if (WIDTH == 1) {
        accumulate_quad_onebit(lo, sh, d, acc);
    } else if (WIDTH == 8) {
        accumulate_quad_bytes(lo, d, acc);
    } else {
        accumulate_quad<STRADDLE>(lo, sh, cd, d, acc);
    }
}

// The same for the [min, max] encoding: value = fma((float)c, step, min), acc <- acc + value.
template <bool STRADDLE>
__device__ __forceinline__ void accumulate_quad_minmax(uint32_t lo, uint32_t sh, uint32_t b, float step,
                                                       float mn, float4& acc) {
    int k[4];
    extract_quad<STRADDLE>(lo, sh, b, k);
    acc.x = acc.x + __builtin_fmaf((float)k[0], step, mn);
    acc.y = acc.y + __builtin_fmaf((float)k[1], step, mn);
    acc.z = acc.z + __builtin_fmaf((float)k[2], step, mn);
    acc.w = acc.w + __builtin_fmaf((float)k[3], step, mn);
}

__device__ __forceinline__ float readlane_f32(float v, uint32_t lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), (int)lane));
}

}  // namespace decode
}  // namespace mqg
