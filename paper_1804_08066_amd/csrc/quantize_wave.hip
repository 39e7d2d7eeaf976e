// Worker side of MQGrad's hot path on gfx950, wavefront-local variant: Quantize(g, K) of
// Algorithm 1 (WorkerIterate), the range-linear K-bit encode of the Section 3.2 footnote, for
// power-of-two buckets.  (Other bucket sizes take the workgroup-cooperative kernel in
// quantize_pack.hip; both produce the same bits.)  The server's re-quantizing step and the
// deterministic [min, max] encoder run on the same decomposition further down.
//
//   a1  per-bucket range  s = max |g|           DPP / swizzle butterfly inside the wave
//       (or the bucket's L2 norm: quad squares in fp32, a fp64 butterfly above them)
//   a2  position on the 2^K-level grid          u = clamp(fma(g, (L/2)/s, L/2), 0, L)
//   a3  stochastic rounding, Philox4x32-10      c = floor(u) + [(h + 1/2)/65536 < frac(u)]
//   a4  dense little-endian bit packing         LDS-staged per wave, 128-bit stores
//
// Work decomposition.  Each 64-lane wave owns a chunk of CH = 256*R consecutive elements and keeps
// it in registers (R float4 per lane: row j of the chunk is the 256 elements the wave loads with
// one float4 per lane), so every gradient byte is read from HBM exactly once.  Buckets of up to CH
// elements live entirely inside one wave: range reduction, the one IEEE division per bucket, the
// rounding and the packing need no workgroup barrier (the lanes of a wave exchange through LDS behind
// wavefront-scope fences).  Larger buckets (WPB = 2 .. 8 waves per bucket) exchange one value per wave
// through LDS behind a single barrier.
//
// The kernel sits close to both of its limits (the vector ALU is busy for about three quarters of
// its HBM-bound duration), so work is moved off the vector ALU where possible: cross-lane exchange through LDS-pipe swizzles, per-bucket
// values through small per-wave LDS tables, bit placement through LDS atomics.

#include "decode.h"
#include "encode.h"
#include "kernels.h"

#include <type_traits>

namespace mqg {
namespace {

using namespace encode;

// lane ^ 1 exchange on the LDS pipe (bit-mode swizzle: and 0x1F, or 0, xor 1): costs no vector-ALU issue
__device__ __forceinline__ uint32_t swap_adjacent(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x041F);
}

// Max over the `seg_lanes` lanes (8, 16, 32 or 64) that share a bucket, for the rows 0, STRIDE,
// 2*STRIDE, ... of a lane at once: stage by stage over all those rows, so that the cross-lane
// exchanges of different rows are in flight together instead of one dependent chain per row.
// Every lane of a segment ends up with the segment's maximum.
template <int R, int STRIDE>
__device__ __forceinline__ void segment_max_rows(uint32_t (&m)[R], uint32_t seg_lanes, uint32_t lane) {
    // The values are bit patterns of non-negative floats, whose order is the order of the unsigned
    // integers: integer max needs no NaN canonicalisation and takes its DPP operand directly.
#pragma unroll
    for (int j = 0; j < R; j += STRIDE) m[j] = max(m[j], dpp_u32<kDppQuadSwap1>(m[j]));
#pragma unroll
    for (int j = 0; j < R; j += STRIDE) m[j] = max(m[j], dpp_u32<kDppQuadSwap2>(m[j]));
#pragma unroll
    for (int j = 0; j < R; j += STRIDE) m[j] = max(m[j], dpp_u32<kDppRowHalfMirror>(m[j]));
    if (seg_lanes >= 16u) {
#pragma unroll
        for (int j = 0; j < R; j += STRIDE) m[j] = max(m[j], dpp_u32<kDppRowMirror>(m[j]));
    }
    if (seg_lanes >= 32u) {
        uint32_t t[R];
#pragma unroll
        for (int j = 0; j < R; j += STRIDE) t[j] = (uint32_t)__builtin_amdgcn_ds_swizzle((int)m[j], kSwizzleXor16);
#pragma unroll
        for (int j = 0; j < R; j += STRIDE) m[j] = max(m[j], t[j]);
    }
    if (seg_lanes >= 64u) {
        uint32_t t[R];
#pragma unroll
        for (int j = 0; j < R; j += STRIDE) t[j] = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((lane ^ 32u) << 2), (int)m[j]);
#pragma unroll
        for (int j = 0; j < R; j += STRIDE) m[j] = max(m[j], t[j]);
    }
}

// The same butterfly as a sum in fp64 (L2 scale).
template <int R, int STRIDE>
__device__ __forceinline__ void segment_sum_rows(double (&q)[R], uint32_t seg_lanes) {
    for (uint32_t mask = 1; mask < seg_lanes; mask <<= 1) {   // uniform trip count
        double t[R];
#pragma unroll
        for (int j = 0; j < R; j += STRIDE) t[j] = __shfl_xor(q[j], (int)mask, 64);
#pragma unroll
        for (int j = 0; j < R; j += STRIDE) q[j] += t[j];
    }
}

// rows per bucket -> compile-time stride
template <int R, int STRIDE = 1>
__device__ __forceinline__ void segment_max_dispatch(uint32_t (&m)[R], uint32_t rpb, uint32_t seg_lanes, uint32_t lane) {
    if (STRIDE >= R || rpb == (uint32_t)STRIDE) {
        segment_max_rows<R, (STRIDE < R ? STRIDE : R)>(m, seg_lanes, lane);
    } else {
        segment_max_dispatch<R, (STRIDE < R ? 2 * STRIDE : R)>(m, rpb, seg_lanes, lane);
    }
}
template <int R, int STRIDE = 1>
__device__ __forceinline__ void segment_sum_dispatch(double (&q)[R], uint32_t rpb, uint32_t seg_lanes) {
    if (STRIDE >= R || rpb == (uint32_t)STRIDE) {
        segment_sum_rows<R, (STRIDE < R ? STRIDE : R)>(q, seg_lanes);
    } else {
        segment_sum_dispatch<R, (STRIDE < R ? 2 * STRIDE : R)>(q, rpb, seg_lanes);
    }
}

// LDS of one workgroup: everything is indexed by wave, so waves never touch each other's entries
// (except wave_max, which is what the WPB > 1 barrier is for).
template <int R, int NW>
struct WaveShared {
    alignas(16) uint32_t words[NW][64 * R + 8];   // packed output of a chunk: 8*R*bits <= 64*R words (+ 1 for a straddling code, + 3 of shift)
    float smax[NW][8 * R];            // per-bucket max |g| of the chunk (<= CH/32 buckets)
    float ainv[NW][8 * R];            // per-bucket (L/2)/s
    float wave_max[NW];               // chunk maximum, for buckets that span several waves
    double ssq[NW][8 * R];            // per-bucket sum of squares of the chunk (L2 scale only)
    double wave_ssq[NW];
};

// ---- phase 1: load the chunk, clear the wave's packing area, publish the bucket maxima -----------
template <int R, int NW>
__device__ __forceinline__ void clear_words(uint32_t lane, uint32_t wave, WaveShared<R, NW>& sm) {
    for (uint32_t i = lane; i < 16u * R; i += 64u) {
        *reinterpret_cast<v4u*>(&sm.words[wave][4u * i]) = v4u{0u, 0u, 0u, 0u};
    }
}

template <int R, int WPB, int NW>
__device__ __forceinline__ void reduce_ranges(const float4 (&x)[R], uint32_t lane, uint32_t wave,
                                              const uint32_t (&slot)[R], uint32_t seg_lanes, uint32_t rpb,
                                              WaveShared<R, NW>& sm, bool l2 = false);

// One Philox call covers 8 consecutive elements = the quads of an even/odd lane pair.  For the row
// pair (jp, jp + 1) the even lane draws for row jp and the odd lane for row jp + 1, so no lane makes a
// call whose output is thrown away.  The numbers depend on the position only, not on the data.
// Returns the complemented words: the rounding consumes 65535 - h.
__device__ __forceinline__ void draw_pair(const QuantizeArgs& a, uint64_t cb, uint32_t lane, int jp, uint32_t (&o)[4]) {
    const uint64_t group0 = (a.elem_base + cb) >> 3;           // both multiples of 8
    const uint32_t my_row = jp + (lane & 1u);
    const uint64_t grp = group0 + (uint64_t)((my_row * 64u + lane) >> 1);
    philox4x32_10<true>((uint32_t)grp, (uint32_t)(grp >> 32), a.iteration, a.worker, a.key0, a.key1, o);
}
template <int R>
struct Draws {
    uint32_t o[R / 2][4];
};

// one HBM pass: the chunk's values into registers
template <int R, bool FULL>
__device__ __forceinline__ void load_chunk(const float* __restrict__ g, uint32_t count, uint32_t lane, float4 (&x)[R]) {
    if (FULL) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f_a4*>(g + 4u * (j * 64u + lane)));
            x[j] = make_float4(t.x, t.y, t.z, t.w);
        }
    } else {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint32_t el = 4u * (j * 64u + lane);
            x[j].x = (el + 0u < count) ? g[el + 0] : 0.0f;
            x[j].y = (el + 1u < count) ? g[el + 1] : 0.0f;
            x[j].z = (el + 2u < count) ? g[el + 2] : 0.0f;
            x[j].w = (el + 3u < count) ? g[el + 3] : 0.0f;
        }
    }
}

// a1: bucket range of the values in registers
template <int R, int WPB, int NW>
__device__ __forceinline__ void reduce_ranges(const float4 (&x)[R], uint32_t lane, uint32_t wave,
                                              const uint32_t (&slot)[R], uint32_t seg_lanes, uint32_t rpb,
                                              WaveShared<R, NW>& sm, bool l2) {
    if (l2) {
        // L2 scale: squares of a quad in fp32, everything above in fp64, in a fixed order
        double q[R];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            q[j] = (double)((x[j].x * x[j].x + x[j].y * x[j].y) + (x[j].z * x[j].z + x[j].w * x[j].w));
        }
#pragma unroll
        for (int step = 1; step < R; step <<= 1) {
            if (rpb > (uint32_t)step) {
#pragma unroll
                for (int j = 0; j + step < R; j += 2 * step) q[j] += q[j + step];
            }
        }
        segment_sum_dispatch<R>(q, rpb, seg_lanes);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (((uint32_t)j & (rpb - 1u)) == 0u && (lane & (seg_lanes - 1u)) == 0u) sm.ssq[wave][slot[j]] = q[j];
        }
        if (WPB > 1 && lane == 0u) sm.wave_ssq[wave] = sm.ssq[wave][0];
    }
    float m[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        m[j] = fmaxf(fmaxf(fabsf(x[j].x), fabsf(x[j].y)), fmaxf(fabsf(x[j].z), fabsf(x[j].w)));
    }
    // fold the rows of one bucket into its first row
#pragma unroll
    for (int step = 1; step < R; step <<= 1) {
        if (rpb > (uint32_t)step) {
#pragma unroll
            for (int j = 0; j + step < R; j += 2 * step) m[j] = fmaxf(m[j], m[j + step]);
        }
    }
    // reduce across the lanes of the bucket; the first lane of each bucket publishes the result
    uint32_t mb[R];
#pragma unroll
    for (int j = 0; j < R; ++j) mb[j] = __builtin_bit_cast(uint32_t, m[j]);   // m >= 0: bit order = value order
    segment_max_dispatch<R>(mb, rpb, seg_lanes, lane);
#pragma unroll
    for (int j = 0; j < R; ++j) {
        if (((uint32_t)j & (rpb - 1u)) == 0u && (lane & (seg_lanes - 1u)) == 0u) {
            sm.smax[wave][slot[j]] = __builtin_bit_cast(float, mb[j]);
        }
    }
    if (WPB > 1 && lane == 0u) sm.wave_max[wave] = sm.smax[wave][0];   // buckets spanning WPB waves
}

// The chunk's packed words from the wave's LDS area to the stream, 128 bits per lane.  The stores carry
// agent scope (write-through to memory, the line stays in L2): measured against streaming and ordinary
// stores at 100 M elements they are 1-3 us faster in this kernel at every width, and the server step
// that follows finds the code words in the last-level cache (8 workers at up to 4 bits are 400 MB or
// less): its time drops by 3-11 %.
// stream_out: the caller said that the code words will not be read from this GPU's caches (several workers'
// streams that together exceed them, or streams that leave the GPU): streaming stores instead.
template <int R, int NW, bool FULL>
__device__ __forceinline__ void store_chunk_words(uint32_t* __restrict__ out, uint32_t count, uint32_t b, uint32_t lane,
                                                  uint32_t wave, const WaveShared<R, NW>& sm, const bool stream_out) {
    if (FULL) {
        for (uint32_t i = lane; i < 2u * R * b; i += 64u) {   // 8*R*bits words = 2*R*bits groups of 4
            const v4u w = *reinterpret_cast<const v4u*>(&sm.words[wave][4u * i]);
            if (stream_out) {
                __builtin_nontemporal_store(w, reinterpret_cast<v4u_a4*>(out + 4u * i));
            } else {
                store_v4u_agent(out, 16u * i, w);
            }
        }
    } else {
        const uint32_t nwords = (count * b + 31u) >> 5;
        for (uint32_t i = lane; i < nwords; i += 64u) out[i] = sm.words[wave][i];
    }
}

// a2..a4 for the chunk's rows: grid position, stochastic rounding, packing into the wave's LDS area.
// sm.ainv[wave][slot[j]] holds the factor of row j's quad.  TAIL: which parts of the chunk can lie past
// `count` -- none, whole quads only (count is a multiple of 4), or single elements.
constexpr int kTailNone = 0, kTailQuads = 1, kTailElements = 2;
template <int R, int NW, int TAIL>
__device__ __forceinline__ void round_and_pack_rows(const QuantizeArgs& a, uint64_t cb, uint32_t count, uint32_t lane,
                                                    uint32_t wave, const uint32_t (&slot)[R], const float4 (&x)[R],
                                                    WaveShared<R, NW>& sm, const FixedGrid& fg, const Draws<R>* drawn,
                                                    const uint32_t word_shift = 0u) {
    // word_shift (0..3): the chunk's word i is kept at sm.words[wave][word_shift + i]
    const uint32_t b = a.bits;
    const uint32_t odd = lane & 1u;
    const uint32_t cell_bit = 4u * b * (lane & 7u);            // this lane's bit offset in its 32-element cell
    const uint32_t sh = cell_bit & 31u;
    const uint32_t word_in_cell = cell_bit >> 5;
    const bool straddle = sh + 4u * b > 32u;

#pragma unroll
    for (int jp = 0; jp < R; jp += 2) {
        // The lane pair's call for rows jp and jp + 1 (made here unless it was made earlier); each lane
        // then takes the half it needs from its partner.  The swaps run with every lane active (a lane
        // swap under a divergent branch would read switched-off partners); the selects that follow
        // keep the half each lane needs.
        uint32_t o[4];
        if (drawn != nullptr) {
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = drawn->o[jp / 2][i];
        } else {
            draw_pair(a, cb, lane, jp, o);
        }
        const uint32_t p0 = swap_adjacent(o[0]), p1 = swap_adjacent(o[1]);
        const uint32_t p2 = swap_adjacent(o[2]), p3 = swap_adjacent(o[3]);
        const uint32_t rw[2][2] = {{odd ? p2 : o[0], odd ? p3 : o[1]},    // row jp: the even lane's call
                                   {odd ? o[2] : p0, odd ? o[3] : p1}};   // row jp+1: the odd lane's call
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int j = jp + t;
            const uint32_t ql = j * 64u + lane;
            const uint32_t el = 4u * ql;
            const float ainv = sm.ainv[wave][slot[j]];
            uint32_t t0 = round_code_hi(x[j].x, ainv, fg, rw[t][0] & 0xFFFFu);
            uint32_t t1 = round_code_hi(x[j].y, ainv, fg, rw[t][0] >> 16);
            uint32_t t2 = round_code_hi(x[j].z, ainv, fg, rw[t][1] & 0xFFFFu);
            uint32_t t3 = round_code_hi(x[j].w, ainv, fg, rw[t][1] >> 16);
            if (TAIL == kTailElements) {   // elements past the end contribute zero bits
                if (el + 0u >= count) t0 = 0u;
                if (el + 1u >= count) t1 = 0u;
                if (el + 2u >= count) t2 = 0u;
                if (el + 3u >= count) t3 = 0u;
            }
            const uint32_t v = pack_quad_hi(t0, t1, t2, t3, b, 2u * b, 3u * b);
            if (TAIL == kTailNone || el < count) {
                const uint32_t w0 = (ql >> 3) * b + word_in_cell + word_shift;
                atomicOr(&sm.words[wave][w0], v << sh);
                if (straddle) atomicOr(&sm.words[wave][w0 + 1u], v >> (32u - sh));
            }
        }
    }
}

// ---- phase 2: scales, grid position, stochastic rounding, packing, store -------------------------
template <int R, int WPB, int NW, bool FULL>
__device__ __forceinline__ void quantize_and_pack(const QuantizeArgs& a, uint64_t cb, uint32_t count, uint32_t lane,
                                                  uint32_t wave, const uint32_t (&slot)[R], uint32_t nbc,
                                                  uint64_t kb_first, const float4 (&x)[R], WaveShared<R, NW>& sm,
                                                  float range_div = 1.0f, const Draws<R>* drawn = nullptr) {
    // range_div: the stored scale is range / range_div (1 for a plain quantize, W for the server's mean)
    const uint32_t b = a.bits;
    const uint32_t shift = (uint32_t)a.bucket_shift;
    const float Lf = (float)((1u << b) - 1u);
    const float halfL = 0.5f * Lf;
    const FixedGrid fg = fixed_grid(b);

    wave_lds_fence();   // the ranges other lanes of this wave published are read below
    if (WPB > 1 && a.scales_in == nullptr && lane == 0u) {
        const uint32_t w0 = wave & ~(uint32_t)(WPB - 1);
        float r = sm.wave_max[w0];
#pragma unroll
        for (int t = 1; t < WPB; ++t) r = fmaxf(r, sm.wave_max[w0 + t]);
        sm.smax[wave][0] = r;
        if (a.scale_mode == MQG_SCALE_L2) {
            double t = sm.wave_ssq[w0];
#pragma unroll
            for (int u = 1; u < WPB; ++u) t += sm.wave_ssq[w0 + u];
            sm.ssq[wave][0] = t;
        }
    }
    // one lane per bucket: floor, store the scale, divide once
    if (lane < nbc) {
        const bool exists = WPB > 1 ? true : ((lane << shift) < count);   // bucket starts inside the vector
        float s = 0.0f;
        if (exists) {
            if (a.scales_in != nullptr) {
                s = a.scales_in[kb_first + lane];
            } else {
                s = sm.smax[wave][lane];
                if (a.scale_mode == MQG_SCALE_L2) {   // the norm, raised to max |g| if rounding left it below
                    const float norm = (float)__builtin_sqrt(sm.ssq[wave][lane]);
                    s = norm < s ? s : norm;
                }
                if (!(s >= 0x1p-96f)) s = 0.0f;
            }
            if (WPB == 1 || (wave & (WPB - 1)) == 0u) a.scales[kb_first + lane] = (range_div == 1.0f) ? s : s / range_div;
        }
        // IEEE-correct fp32 division, once per bucket; the factor is kept times 2^16 (exact) for the
        // fixed-point rounding
        sm.ainv[wave][lane] = (s > 0.0f) ? (halfL / s) * 65536.0f : 0.0f;
    }
    wave_lds_fence();   // every lane reads its buckets' factors; the packing area was cleared by other lanes

    round_and_pack_rows<R, NW, FULL ? kTailNone : kTailElements>(a, cb, count, lane, wave, slot, x, sm, fg, drawn);

    // store the chunk's words
    wave_lds_fence();   // a word holds bits placed by several lanes
    uint32_t* __restrict__ out = a.packed + (cb >> 5) * b;
    store_chunk_words<R, NW, FULL>(out, count, b, lane, wave, sm, a.stream_codes != 0u);
}

// A wave's chunk and how buckets lie in it.  WPB == 1: the chunk holds nbc = CH / bucket whole buckets; a
// bucket is `seg_lanes` lanes of one row (bucket <= 256) or `rpb` whole rows (bucket >= 256).  WPB > 1:
// the chunk is part of one bucket.
template <int R>
struct ChunkShape {
    uint32_t lane, wave;   // wave: uniform (read with v_readfirstlane), so what follows from it is scalar work
    uint64_t chunk, cb;    // chunk index; first element of the chunk
    bool active, full;     // the chunk starts inside the tensor; it lies inside it entirely
    uint32_t count;        // elements of the chunk inside the tensor
    uint32_t nbc;          // buckets per chunk
    uint32_t seg_lanes;    // lanes of a row that share a bucket
    uint32_t rpb;          // rows per bucket
    uint64_t kb_first;     // global index of the chunk's first bucket
};
// bucket (chunk-local) of row j's quad
template <int R, int WPB>
__device__ __forceinline__ void chunk_slots(const QuantizeArgs& a, uint32_t lane, uint32_t (&slot)[R]) {
#pragma unroll
    for (int j = 0; j < R; ++j) slot[j] = WPB > 1 ? 0u : ((4u * (j * 64u + lane)) >> (uint32_t)a.bucket_shift);
}
template <int R, int WPB, int NW>
__device__ __forceinline__ ChunkShape<R> chunk_shape(const QuantizeArgs& a, const uint64_t block) {
    constexpr uint32_t CH = 256u * R;
    static_assert(NW % WPB == 0, "the waves of a bucket share a workgroup");
    ChunkShape<R> c;
    const uint32_t tid = threadIdx.x;
    c.lane = tid & 63u;
    c.wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6));
    c.chunk = block * NW + c.wave;
    c.cb = c.chunk * CH;
    c.active = c.cb < a.n;   // waves past the end only keep the barrier company
    c.count = !c.active ? 0u : (a.n - c.cb < CH ? (uint32_t)(a.n - c.cb) : CH);
    c.full = c.count == CH;
    const uint32_t shift = (uint32_t)a.bucket_shift;   // log2(bucket), >= 5
    c.nbc = WPB > 1 ? 1u : (CH >> shift);
    c.seg_lanes = (WPB > 1 || shift >= 8u) ? 64u : (1u << (shift - 2u));
    c.rpb = WPB > 1 ? (uint32_t)R : (shift >= 8u ? (1u << (shift - 8u)) : 1u);
    c.kb_first = WPB > 1 ? (c.chunk / WPB) : (c.cb >> shift);
    return c;
}

// R: float4 per lane; WPB: waves per bucket (1: bucket <= CH; otherwise bucket = WPB*CH);
// NW: waves per workgroup, a multiple of WPB
// HOIST: the Philox calls of the chunk are made before the range reduction and its barrier (they depend
// on the position only) and kept in 2*R registers until the rounding.
template <int R, int WPB, int NW, bool HOIST>
__device__ __forceinline__ void quantize_wave_block(const QuantizeArgs& a, const uint64_t block, WaveShared<R, NW>& sm) {
    const ChunkShape<R> c = chunk_shape<R, WPB, NW>(a, block);
    const uint32_t lane = c.lane, wave = c.wave;
    uint32_t slot[R];
    chunk_slots<R, WPB>(a, lane, slot);

    float4 x[R];
    if (c.full) {
        load_chunk<R, true>(a.grad + c.cb, c.count, lane, x);
    } else {
        load_chunk<R, false>(a.grad + c.cb, c.count, lane, x);
    }
    // while the loads are in flight: clear the wave's packing area; when asked to, draw the chunk's
    // random numbers ahead of the barrier
    clear_words<R, NW>(lane, wave, sm);
    Draws<R> draws;
    if (HOIST) {
#pragma unroll
        for (int jp = 0; jp < R; jp += 2) draw_pair(a, c.cb, lane, jp, draws.o[jp / 2]);
    }
    if (a.scales_in == nullptr) {
        reduce_ranges<R, WPB, NW>(x, lane, wave, slot, c.seg_lanes, c.rpb, sm, a.scale_mode == MQG_SCALE_L2);
    }
    if (WPB > 1) __syncthreads();   // every wave of the group arrives here exactly once
    if (!c.active) return;
    const Draws<R>* drawn = HOIST ? &draws : nullptr;
    if (c.full) {
        quantize_and_pack<R, WPB, NW, true>(a, c.cb, c.count, lane, wave, slot, c.nbc, c.kb_first, x, sm, 1.0f, drawn);
    } else {
        quantize_and_pack<R, WPB, NW, false>(a, c.cb, c.count, lane, wave, slot, c.nbc, c.kb_first, x, sm, 1.0f, drawn);
    }
}

// OCC: cap on the waves per SIMD (8 = none).  The 2048-element shape fits six waves per SIMD; that is
// faster than five up to 3 bits and slower from 4 bits on, where a wave writes more (measured at 100 M
// elements, buckets 128 and 1024: -2..-4 us and +1..+3 us), so the launch picks the cap by the width.
template <int R, int WPB, int NW, int OCC, bool HOIST>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(1, OCC))) void quantize_wave_kernel(const QuantizeArgs a) {
    __shared__ WaveShared<R, NW> sm;
    quantize_wave_block<R, WPB, NW, HOIST>(a, blockIdx.x, sm);
}

// Several layer tensors of one worker in one launch: workgroup -> (tensor, block of the tensor) through
// the prefix table of block counts.
template <int R, int WPB, int NW, int OCC, bool HOIST>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(1, OCC))) void quantize_tensors_wave_kernel(const BatchQuantizeArgs ba) {
    __shared__ WaveShared<R, NW> sm;
    uint32_t lo = 0, hi = ba.count;          // tile_start[lo] <= blockIdx.x < tile_start[hi]
    while (hi - lo > 1u) {
        const uint32_t mid = (lo + hi) >> 1;
        if (blockIdx.x >= ba.tile_start[mid]) lo = mid; else hi = mid;
    }
    QuantizeArgs a = ba.common;
    a.grad = ba.t[lo].grad;
    a.n = ba.t[lo].n;
    a.elem_base = ba.t[lo].elem_base;
    a.packed = ba.t[lo].packed;
    a.scales = ba.t[lo].scales;
    a.scales_in = ba.t[lo].scales_in;
    quantize_wave_block<R, WPB, NW, HOIST>(a, blockIdx.x - ba.tile_start[lo], sm);
}

// ---- buckets of any whole number of cells ------------------------------------------------------------
// Bucket sizes that are multiples of 32 but not powers of two (96 .. 4064 elements).  A workgroup owns a
// tile of whole buckets, as many as fit into NW * 2048 elements; the tile's 32-element cells are dealt out
// to the waves in equal runs (a run is at most 64 cells, one per 8 lanes and row), so a bucket may lie in
// two or more waves: the cells' maxima meet in one LDS slot per bucket (integer max on the bit patterns),
// between the workgroup's two barriers.  The first barrier falls while the loads are in flight.
// Everything after the second -- the bucket factors a wave needs, rounding, packing, stores -- is
// wave-local as in the kernel above.
struct CellGeometry {
    uint32_t bucket_cells;     // cells per bucket: bucket / 32, 3 .. 127
    uint32_t tile_buckets;     // whole buckets per tile
    uint32_t tile_cells;       // bucket_cells * tile_buckets <= NW * 64
    uint32_t cells_per_wave;   // ceil(tile_cells / NW) <= 64
    uint32_t magic;            // ceil(65536 / bucket_cells): (cell * magic) >> 16 = cell / bucket_cells for cell < 512
};

template <int NW>
struct CellShared {
    uint32_t bmax[NW * 64 / 3 + 1];   // per bucket of the tile: bit pattern of max |g|
};

template <int NW, bool HOIST>
__device__ __forceinline__ void quantize_cells_block(const QuantizeArgs& a, const CellGeometry& g, const uint64_t tile,
                                                     WaveShared<8, NW>& sm, CellShared<NW>& cs) {
    constexpr int R = 8;
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6));
    const uint64_t tile_base = tile * ((uint64_t)g.tile_cells * 32u);          // first element of the tile (< n)
    const uint32_t cell0 = wave * g.cells_per_wave;                             // the wave's run of cells
    const uint32_t ncell = cell0 >= g.tile_cells ? 0u : (g.tile_cells - cell0 < g.cells_per_wave ? g.tile_cells - cell0 : g.cells_per_wave);
    const uint64_t cb = tile_base + 32u * cell0;                                // first element of the run
    const uint32_t count = (ncell == 0u || cb >= a.n) ? 0u : (a.n - cb < 32u * ncell ? (uint32_t)(a.n - cb) : 32u * ncell);
    const bool whole_quads = (count & 3u) == 0u;   // always, except for the run that holds the tensor's ragged end

    float4 x[R];
    if (whole_quads) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint32_t el = 4u * (j * 64u + lane);
            if (el < count) {
                const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f_a4*>(a.grad + cb + el));
                x[j] = make_float4(t.x, t.y, t.z, t.w);
            } else {
                x[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
        }
    } else {
        load_chunk<R, false>(a.grad + cb, count, lane, x);
    }
    // while the loads are in flight
    clear_words<R, NW>(lane, wave, sm);
    if (lane == 0u) *reinterpret_cast<v4u*>(&sm.words[wave][64u * R]) = v4u{0u, 0u, 0u, 0u};   // the run's words may sit up to three further on
    for (uint32_t i = tid; i < g.tile_buckets; i += 64u * NW) cs.bmax[i] = 0u;
    Draws<R> draws;
    if (HOIST) {
#pragma unroll
        for (int jp = 0; jp < R; jp += 2) draw_pair(a, cb, lane, jp, draws.o[jp / 2]);
    }
    // tile-local bucket of row j's cell; rows past the run point at buckets that are never used
    uint32_t kb[R];
#pragma unroll
    for (int j = 0; j < R; ++j) kb[j] = ((cell0 + 8u * j + (lane >> 3)) * g.magic) >> 16;
    __syncthreads();

    if (a.scales_in == nullptr) {
        uint32_t m[R];   // bit patterns of non-negative floats: integer order = value order
#pragma unroll
        for (int j = 0; j < R; ++j) {
            m[j] = __builtin_bit_cast(uint32_t, fmaxf(fmaxf(fabsf(x[j].x), fabsf(x[j].y)), fmaxf(fabsf(x[j].z), fabsf(x[j].w))));
        }
#pragma unroll
        for (int j = 0; j < R; ++j) m[j] = max(m[j], dpp_u32<kDppQuadSwap1>(m[j]));
#pragma unroll
        for (int j = 0; j < R; ++j) m[j] = max(m[j], dpp_u32<kDppQuadSwap2>(m[j]));
#pragma unroll
        for (int j = 0; j < R; ++j) m[j] = max(m[j], dpp_u32<kDppRowHalfMirror>(m[j]));
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if ((lane & 7u) == 0u && 8u * j + (lane >> 3) < ncell) atomicMax(&cs.bmax[kb[j]], m[j]);
        }
    }
    __syncthreads();
    if (count == 0u) return;

    // the buckets this run touches: kbw0 .. kbw0 + nbw - 1 (nbw <= 64 / 3 + 2); one lane each
    const uint32_t kbw0 = (cell0 * g.magic) >> 16;
    const uint32_t nbw = (((cell0 + ncell - 1u) * g.magic) >> 16) - kbw0 + 1u;
    const uint32_t b = a.bits;
    const float halfL = 0.5f * (float)((1u << b) - 1u);
    if (lane < nbw) {
        const uint32_t k = kbw0 + lane;
        const uint64_t kg = tile * g.tile_buckets + k;                                    // global bucket index
        const bool exists = tile_base + (uint64_t)k * a.bucket < a.n;                     // the bucket starts inside the tensor
        float s = 0.0f;
        if (exists) {
            if (a.scales_in != nullptr) {
                s = a.scales_in[kg];
            } else {
                s = __builtin_bit_cast(float, cs.bmax[k]);
                if (!(s >= 0x1p-96f)) s = 0.0f;
            }
            if (k * g.bucket_cells >= cell0) a.scales[kg] = s;   // the run that holds the bucket's first cell stores it
        }
        sm.ainv[wave][lane] = (s > 0.0f) ? (halfL / s) * 65536.0f : 0.0f;   // IEEE-correct fp32 division, times 2^16 (exact)
    }
    uint32_t slot[R];
#pragma unroll
    for (int j = 0; j < R; ++j) slot[j] = kb[j] - kbw0;   // < 64 / 3 + 2 + 64 / 3: inside sm.ainv[wave]
    wave_lds_fence();

    const FixedGrid fg = fixed_grid(b);
    const Draws<R>* drawn = HOIST ? &draws : nullptr;
    // The run's words start at any word of the stream.  They are kept in LDS shifted by the stream
    // position modulo four, so that 16-byte groups of the stream are 16-byte groups in LDS: up to three
    // single words, then 128-bit stores at aligned addresses (unaligned ones cost 10 % of the kernel's
    // time), then up to three single words.  Every store carries the same agent scope: ordinary stores
    // into cache lines that also receive agent-scope stores slowed the kernel from 72 to 128 us.
    const uint64_t word0 = (cb >> 5) * b;
    const uint32_t shift4 = (uint32_t)word0 & 3u;
    if (whole_quads) {
        round_and_pack_rows<R, NW, kTailQuads>(a, cb, count, lane, wave, slot, x, sm, fg, drawn, shift4);
    } else {
        round_and_pack_rows<R, NW, kTailElements>(a, cb, count, lane, wave, slot, x, sm, fg, drawn, shift4);
    }
    wave_lds_fence();   // a word holds bits placed by several lanes

    const uint32_t nwords = (count * b + 31u) >> 5;
    const uint32_t* __restrict__ lw = sm.words[wave];                 // stream word word0 + i is lw[shift4 + i]
    uint32_t* __restrict__ out = a.packed + (word0 - shift4);         // 16-byte aligned when a.packed is; out[shift4 + i] is stream word word0 + i
    const uint32_t first = shift4, last = shift4 + nwords;            // the run in units of `out` / `lw` words
    const uint32_t body0 = (first + 3u) & ~3u;                        // first aligned group
    const uint32_t body1 = last & ~3u;                                // end of the last whole group
    if (a.stream_codes != 0u) {   // the same stores with the streaming hint (see store_chunk_words)
        if (body0 < body1) {
            if (first + lane < body0) __builtin_nontemporal_store(lw[first + lane], out + first + lane);
            for (uint32_t i = (body0 >> 2) + lane; i < (body1 >> 2); i += 64u) {
                __builtin_nontemporal_store(*reinterpret_cast<const v4u*>(&lw[4u * i]), reinterpret_cast<v4u_a4*>(out + 4u * i));
            }
            if (body1 + lane < last) __builtin_nontemporal_store(lw[body1 + lane], out + body1 + lane);
        } else if (first + lane < last) {
            __builtin_nontemporal_store(lw[first + lane], out + first + lane);
        }
    } else if (body0 < body1) {
        if (first + lane < body0) store_u32_agent(out, 4u * (first + lane), lw[first + lane]);
        for (uint32_t i = (body0 >> 2) + lane; i < (body1 >> 2); i += 64u) {
            store_v4u_agent(out, 16u * i, *reinterpret_cast<const v4u*>(&lw[4u * i]));
        }
        if (body1 + lane < last) store_u32_agent(out, 4u * (body1 + lane), lw[body1 + lane]);
    } else if (first + lane < last) {   // fewer than seven words and no whole group
        store_u32_agent(out, 4u * (first + lane), lw[first + lane]);
    }
}

template <int NW, int OCC, bool HOIST>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(1, OCC))) void quantize_cells_kernel(const QuantizeArgs a, const CellGeometry g) {
    __shared__ WaveShared<8, NW> sm;
    __shared__ CellShared<NW> cs;
    quantize_cells_block<NW, HOIST>(a, g, blockIdx.x, sm, cs);
}

// Several layer tensors of one worker in one launch, as quantize_tensors_wave_kernel maps them.
template <int NW, int OCC, bool HOIST>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(1, OCC))) void quantize_tensors_cells_kernel(const BatchQuantizeArgs ba, const CellGeometry g) {
    __shared__ WaveShared<8, NW> sm;
    __shared__ CellShared<NW> cs;
    uint32_t lo = 0, hi = ba.count;          // tile_start[lo] <= blockIdx.x < tile_start[hi]
    while (hi - lo > 1u) {
        const uint32_t mid = (lo + hi) >> 1;
        if (blockIdx.x >= ba.tile_start[mid]) lo = mid; else hi = mid;
    }
    QuantizeArgs a = ba.common;
    a.grad = ba.t[lo].grad;
    a.n = ba.t[lo].n;
    a.elem_base = ba.t[lo].elem_base;
    a.packed = ba.t[lo].packed;
    a.scales = ba.t[lo].scales;
    a.scales_in = ba.t[lo].scales_in;
    quantize_cells_block<NW, HOIST>(a, g, blockIdx.x - ba.tile_start[lo], sm, cs);
}

// ---- the server's re-quantizing step on the same decomposition -------------------------------------
// ReceiveQGThenSendQG of Algorithm 1: the chunk's values are not loaded but decoded -- the sum over the
// W workers' de-quantized gradients, the ordered fma chain of the fused update -- and then quantized
// exactly as a gradient would be; the stored range is divided by W.  Buckets of 128 elements and more:
// a wave's 256-element row lies in one bucket (two at bucket 128), so the bucket steps of the chunk are
// divided once by a few lanes and the worker loop broadcasts them with v_readlane (no LDS table, no
// barrier).
// RPB: rows of the chunk per bucket (bucket = 256 * RPB when WPB == 1; R when the chunk is part of one
// bucket), a compile-time number so that rows of one bucket share one division and one v_readlane per
// worker.  RPB = 0 stands for bucket 128: a row is two buckets, lanes 0-31 and 32-63 select their step.
// LUT = 1 .. 4: the decode takes (float)(2c - L) from a table in LDS (decode::accumulate_quad_lut; the
// workgroup fills it first, one barrier) -- half the vector operations of the arithmetic decode per
// code, and this step is bound by their issue.
template <int R, int WPB, int NW, int RPB, bool STRADDLE, bool ONCE, int WIDTH, int LUT = 0>
__global__ __launch_bounds__(64 * NW) void requantize_wave_kernel(const RequantArgs ra) {
    constexpr uint32_t CH = 256u * R;
    constexpr int kChunk = 32 / R;   // workers whose code loads are in flight together
    static_assert(NW % WPB == 0, "the waves of a bucket share a workgroup");
    __shared__ WaveShared<R, NW> sm;
    __shared__ __attribute__((aligned(16))) float lut[LUT > 0 ? decode::kLutFloats : 1];
    const QuantizeArgs& a = ra.q;

    const uint32_t tid = threadIdx.x;
    if (LUT > 0) {
        decode::build_pair_lut(lut, a.bits, tid, 64u * NW);
        __syncthreads();
    }
    const uint32_t lane = tid & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6));   // uniform: what follows from it is scalar work
    const uint64_t chunk = (uint64_t)blockIdx.x * NW + wave;
    const uint64_t cb = chunk * CH;
    const bool active = cb < a.n;
    const uint32_t count = !active ? 0u : (a.n - cb < CH ? (uint32_t)(a.n - cb) : CH);
    const bool full = count == CH;

    const uint32_t shift = (uint32_t)a.bucket_shift;                      // log2(bucket), >= 7 here
    constexpr bool HALF = RPB == 0;                                        // bucket 128: two buckets per row
    constexpr int RP = HALF ? 1 : RPB;
    static_assert(HALF ? (WPB == 1 && R == 4) : (R % RP == 0 && (WPB == 1 || RPB == R)),
                  "whole buckets per chunk, or one bucket over several chunks");
    constexpr uint32_t nbc = HALF ? 2u * R : R / RP;                       // buckets per chunk
    constexpr uint32_t rpb = RP;                                           // rows per bucket
    constexpr uint32_t seg_lanes = HALF ? 32u : 64u;                       // lanes of a row per bucket
    const uint64_t kb_first = WPB > 1 ? (chunk / WPB) : chunk * nbc;       // global index of the chunk's first bucket
    uint32_t slot[R];
#pragma unroll
    for (int j = 0; j < R; ++j) slot[j] = HALF ? 2u * j + (lane >> 5) : (uint32_t)(j / RP);   // bucket of row j's quad

    float4 x[R];
#pragma unroll
    for (int j = 0; j < R; ++j) x[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (active) {
        const uint32_t b = a.bits;
        const decode::Centred cd = decode::centred(b);
        const float Lf = (float)((1u << b) - 1u);
        const uint64_t nb_total = (a.n + a.bucket - 1u) >> shift;
        // Bucket 128 -- eight buckets per chunk and eight workers per worker chunk: lane l takes (worker
        // l / 8 of the worker chunk, bucket l % 8), one division per lane; the decode reads the two steps
        // of a row back with v_readlane and each half of the wave selects its own.  The first scale is
        // requested ahead of the code words: loads return in order, so the wait for it does not have
        // to drain the code loads behind it.
        static_assert(!HALF || kChunk * nbc == 64u, "one (worker, bucket) pair per lane");
        uint64_t my_kb = kb_first + (lane % nbc);
        if (my_kb >= nb_total) my_kb = nb_total - 1u;   // bucket past the end
        const auto my_scale = [&](uint32_t w0) {
            const uint32_t w = w0 + lane / nbc;
            return ra.scales[w < ra.W ? w : 0u][my_kb];
        };
        float sw = HALF ? my_scale(0u) : 0.0f;
        const decode::CodeWindows<R> cw = decode::code_windows<R, 64>(a.n, cb, b, lane);
        decode::CodeRegs<R, kChunk> c;
        decode::fetch_codes<R, kChunk, ONCE>(ra.packed, ra.W, 0u, cw, c);
        clear_words<R, NW>(lane, wave, sm);   // while the loads are in flight
        if (HALF) {
            const bool second = lane >= 32u;
            for (uint32_t w0 = 0; w0 < ra.W; w0 += kChunk) {
                if (w0 > 0) {
                    sw = my_scale(w0);
                    decode::fetch_codes<R, kChunk, ONCE>(ra.packed, ra.W, w0, cw, c);
                }
                const float dl = sw / Lf;   // IEEE-correct fp32 division
#pragma unroll
                for (int t = 0; t < kChunk; ++t) {
                    if (w0 + t < ra.W) {
#pragma unroll
                        for (int j = 0; j < R; ++j) {
                            const float d0 = decode::readlane_f32(dl, t * nbc + 2u * j);
                            const float d1 = decode::readlane_f32(dl, t * nbc + 2u * j + 1u);
                            if (LUT > 0) decode::accumulate_quad_lut<LUT>(c.lo[t][j], cw.sh, lut, second ? d1 : d0, x[j]);
                            else decode::accumulate_quad_w<STRADDLE, WIDTH>(c.lo[t][j], cw.sh, cd, second ? d1 : d0, x[j]);
                        }
                    }
                }
            }
        } else {
            // lane w: worker w's step of each bucket of the chunk
            const float* my_scales = ra.scales[lane < ra.W ? lane : 0u];
            float d[R];
#pragma unroll
            for (int j = 0; j < R; ++j) {
                uint64_t kb = kb_first + slot[j];
                if (kb >= nb_total) kb = nb_total - 1u;   // row past the end
                d[j] = my_scales[kb] / Lf;                // IEEE-correct fp32 division
            }
            for (uint32_t w0 = 0; w0 < ra.W; w0 += kChunk) {
                if (w0 > 0) decode::fetch_codes<R, kChunk, ONCE>(ra.packed, ra.W, w0, cw, c);
#pragma unroll
                for (int t = 0; t < kChunk; ++t) {
                    if (w0 + t < ra.W) {
#pragma unroll
                        for (int j = 0; j < R; ++j) {
                            const float dw = decode::readlane_f32(d[j], w0 + t);
                            if (LUT > 0) decode::accumulate_quad_lut<LUT>(c.lo[t][j], cw.sh, lut, dw, x[j]);
                            else decode::accumulate_quad_w<STRADDLE, WIDTH>(c.lo[t][j], cw.sh, cd, dw, x[j]);
                        }
                    }
                }
            }
        }
        if (!full) {   // elements past the end decode clamped words: they must not reach the range
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const uint32_t el = 4u * (j * 64u + lane);
                if (el + 0u >= count) x[j].x = 0.0f;
                if (el + 1u >= count) x[j].y = 0.0f;
                if (el + 2u >= count) x[j].z = 0.0f;
                if (el + 3u >= count) x[j].w = 0.0f;
            }
        }
    }
    reduce_ranges<R, WPB, NW>(x, lane, wave, slot, seg_lanes, rpb, sm, a.scale_mode == MQG_SCALE_L2);
    if (WPB > 1) __syncthreads();   // every wave of the group arrives here exactly once
    if (!active) return;
    const float Wf = (float)ra.W;
    if (full) {
        quantize_and_pack<R, WPB, NW, true>(a, cb, count, lane, wave, slot, nbc, kb_first, x, sm, Wf);
    } else {
        quantize_and_pack<R, WPB, NW, false>(a, cb, count, lane, wave, slot, nbc, kb_first, x, sm, Wf);
    }
}

template <int R, int WPB, int NW, int RPB = R>
hipError_t launch_requant_wave(const RequantArgs& ra, hipStream_t stream) {
    const uint64_t per_group = (uint64_t)NW * 256u * R;
    const uint64_t groups = (ra.q.n + per_group - 1) / per_group;
    if (groups > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)groups), block(64 * NW);
    // 1 .. 4 bits: multipliers from a table in LDS (bucket 1024, 8 workers, 100 M elements: 120 / 138 / 151 /
    // 141 us with the arithmetic decode, 100 / 98 / 122 / 122 us with the table)
    if (ra.q.bits == 1u) {
        hipLaunchKernelGGL((requantize_wave_kernel<R, WPB, NW, RPB, false, false, 0, 1>), grid, block, 0, stream, ra);
    } else if (ra.q.bits == 2u) {
        hipLaunchKernelGGL((requantize_wave_kernel<R, WPB, NW, RPB, false, false, 0, 2>), grid, block, 0, stream, ra);
    } else if (ra.q.bits == 3u) {
        hipLaunchKernelGGL((requantize_wave_kernel<R, WPB, NW, RPB, true, false, 0, 3>), grid, block, 0, stream, ra);
    } else if (ra.q.bits == 4u) {
        hipLaunchKernelGGL((requantize_wave_kernel<R, WPB, NW, RPB, false, true, 0, 4>), grid, block, 0, stream, ra);
    } else if (ra.q.bits == 8u) {   // a code is a byte: three-operation decode
        hipLaunchKernelGGL((requantize_wave_kernel<R, WPB, NW, RPB, false, true, 8>), grid, block, 0, stream, ra);
    } else {                        // 5, 6, 7 bits: a quad may spill into the next word; streaming loads
        hipLaunchKernelGGL((requantize_wave_kernel<R, WPB, NW, RPB, true, true, 0>), grid, block, 0, stream, ra);
    }
    return hipGetLastError();
}

// ---- the deterministic [min, max] encoder on the same decomposition ----------------------------------
// The footnote of Section 3.2 read literally: per bucket mn = min g, mx = max g, 2^K - 1 equal steps,
// nearest level (rint), no random numbers.  Same chunks, same packing; the range is a pair, reduced on
// order-preserving integer keys (the minimum as the maximum of the complemented key, so both run
// through the same butterfly).  a.scales receives (mn, mx) pairs; a.scales_in != nullptr gives ONE
// pair for every element (the whole-tensor range computed by an earlier pass).
template <int R, int NW>
struct WaveLows {
    float lo[NW][8 * R];   // per bucket: key of the minimum, then the minimum itself
    float wave_lo[NW];     // chunk minimum key, for buckets that span several waves
};

template <int R, int WPB, int NW, bool FULL>
__device__ __forceinline__ void reduce_minmax(const float4 (&x)[R], uint32_t count, uint32_t lane, uint32_t wave,
                                              const uint32_t (&slot)[R], uint32_t seg_lanes, uint32_t rpb,
                                              WaveShared<R, NW>& sm, WaveLows<R, NW>& lw) {
    const float inf = __builtin_inff();
    float lo[R], hi[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        if (FULL) {
            lo[j] = fminf(fminf(x[j].x, x[j].y), fminf(x[j].z, x[j].w));
            hi[j] = fmaxf(fmaxf(x[j].x, x[j].y), fmaxf(x[j].z, x[j].w));
        } else {   // elements past the end take no part
            const uint32_t el = 4u * (j * 64u + lane);
            const bool v0 = el + 0u < count, v1 = el + 1u < count, v2 = el + 2u < count, v3 = el + 3u < count;
            lo[j] = fminf(fminf(v0 ? x[j].x : inf, v1 ? x[j].y : inf), fminf(v2 ? x[j].z : inf, v3 ? x[j].w : inf));
            hi[j] = fmaxf(fmaxf(v0 ? x[j].x : -inf, v1 ? x[j].y : -inf), fmaxf(v2 ? x[j].z : -inf, v3 ? x[j].w : -inf));
        }
    }
    // fold the rows of one bucket into its first row
#pragma unroll
    for (int step = 1; step < R; step <<= 1) {
        if (rpb > (uint32_t)step) {
#pragma unroll
            for (int j = 0; j + step < R; j += 2 * step) {
                lo[j] = fminf(lo[j], lo[j + step]);
                hi[j] = fmaxf(hi[j], hi[j + step]);
            }
        }
    }
    uint32_t kh[R], nl[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        kh[j] = order_key(hi[j]);
        nl[j] = ~order_key(lo[j]);
    }
    segment_max_dispatch<R>(kh, rpb, seg_lanes, lane);
    segment_max_dispatch<R>(nl, rpb, seg_lanes, lane);
#pragma unroll
    for (int j = 0; j < R; ++j) {
        if (((uint32_t)j & (rpb - 1u)) == 0u && (lane & (seg_lanes - 1u)) == 0u) {
            sm.smax[wave][slot[j]] = __builtin_bit_cast(float, kh[j]);
            lw.lo[wave][slot[j]] = __builtin_bit_cast(float, ~nl[j]);
        }
    }
    if (WPB > 1 && lane == 0u) {   // buckets spanning WPB waves
        sm.wave_max[wave] = sm.smax[wave][0];
        lw.wave_lo[wave] = lw.lo[wave][0];
    }
}

template <int R, int WPB, int NW, bool FULL>
__device__ __forceinline__ void encode_minmax_and_pack(const QuantizeArgs& a, uint64_t cb, uint32_t count, uint32_t lane,
                                                       uint32_t wave, const uint32_t (&slot)[R], uint32_t nbc,
                                                       uint64_t kb_first, const float4 (&x)[R], WaveShared<R, NW>& sm,
                                                       WaveLows<R, NW>& lw) {
    const uint32_t b = a.bits;
    const uint32_t shift = (uint32_t)a.bucket_shift;
    const float Lf = (float)((1u << b) - 1u);
    const bool given = a.scales_in != nullptr;

    wave_lds_fence();   // the keys other lanes of this wave published are read below
    if (WPB > 1 && !given && lane == 0u) {
        const uint32_t w0 = wave & ~(uint32_t)(WPB - 1);
        uint32_t kh = __builtin_bit_cast(uint32_t, sm.wave_max[w0]), kl = __builtin_bit_cast(uint32_t, lw.wave_lo[w0]);
#pragma unroll
        for (int t = 1; t < WPB; ++t) {
            kh = max(kh, __builtin_bit_cast(uint32_t, sm.wave_max[w0 + t]));
            kl = min(kl, __builtin_bit_cast(uint32_t, lw.wave_lo[w0 + t]));
        }
        sm.smax[wave][0] = __builtin_bit_cast(float, kh);
        lw.lo[wave][0] = __builtin_bit_cast(float, kl);
    }
    // one lane per bucket: the range, its store, one division
    if (lane < nbc) {
        const bool exists = WPB > 1 ? true : ((lane << shift) < count);   // bucket starts inside the vector
        float mn = 0.0f, mx = 0.0f;
        if (exists) {
            if (given) {
                mn = a.scales_in[0];
                mx = a.scales_in[1];
            } else {
                mn = key_value(__builtin_bit_cast(uint32_t, lw.lo[wave][lane]));
                mx = key_value(__builtin_bit_cast(uint32_t, sm.smax[wave][lane]));
                if (mn == 0.0f) mn = 0.0f;   // a zero bound is stored as +0
                if (mx == 0.0f) mx = 0.0f;
                if (WPB == 1 || (wave & (WPB - 1)) == 0u) {
                    a.scales[2u * (kb_first + lane)] = mn;
                    a.scales[2u * (kb_first + lane) + 1u] = mx;
                }
            }
        }
        const float r = mx - mn;
        lw.lo[wave][lane] = mn;
        sm.ainv[wave][lane] = (r >= 0x1p-96f) ? Lf / r : 0.0f;   // IEEE-correct fp32 division, once per bucket
    }
    wave_lds_fence();   // every lane reads its buckets' (mn, a); the packing area was cleared by other lanes

    const uint32_t cell_bit = 4u * b * (lane & 7u);            // this lane's bit offset in its 32-element cell
    const uint32_t sh = cell_bit & 31u;
    const uint32_t word_in_cell = cell_bit >> 5;
    const bool straddle = sh + 4u * b > 32u;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t ql = j * 64u + lane;
        const uint32_t el = 4u * ql;
        const float mn = lw.lo[wave][slot[j]], ai = sm.ainv[wave][slot[j]];
        // fmaxf drops a NaN position to 0; positions are integers after rint
        uint32_t k0 = (uint32_t)fminf(fmaxf(__builtin_rintf((x[j].x - mn) * ai), 0.0f), Lf);
        uint32_t k1 = (uint32_t)fminf(fmaxf(__builtin_rintf((x[j].y - mn) * ai), 0.0f), Lf);
        uint32_t k2 = (uint32_t)fminf(fmaxf(__builtin_rintf((x[j].z - mn) * ai), 0.0f), Lf);
        uint32_t k3 = (uint32_t)fminf(fmaxf(__builtin_rintf((x[j].w - mn) * ai), 0.0f), Lf);
        if (!FULL) {   // elements past the end contribute zero bits
            if (el + 0u >= count) k0 = 0u;
            if (el + 1u >= count) k1 = 0u;
            if (el + 2u >= count) k2 = 0u;
            if (el + 3u >= count) k3 = 0u;
        }
        const uint32_t v = (((((k3 << b) | k2) << b) | k1) << b) | k0;
        if (FULL || el < count) {
            const uint32_t w0 = (ql >> 3) * b + word_in_cell;
            atomicOr(&sm.words[wave][w0], v << sh);
            if (straddle) atomicOr(&sm.words[wave][w0 + 1u], v >> (32u - sh));
        }
    }

    wave_lds_fence();   // a word holds bits placed by several lanes
    uint32_t* __restrict__ out = a.packed + (cb >> 5) * b;
    store_chunk_words<R, NW, FULL>(out, count, b, lane, wave, sm, a.stream_codes != 0u);
}

template <int R, int WPB, int NW>
__device__ __forceinline__ void quantize_minmax_wave_block(const QuantizeArgs& a, const uint32_t block, WaveShared<R, NW>& sm,
                                                           WaveLows<R, NW>& lw) {
    const ChunkShape<R> c = chunk_shape<R, WPB, NW>(a, block);
    const uint32_t lane = c.lane, wave = c.wave;
    uint32_t slot[R];
    chunk_slots<R, WPB>(a, lane, slot);

    float4 x[R];
    if (c.full) {
        load_chunk<R, true>(a.grad + c.cb, c.count, lane, x);
    } else {
        load_chunk<R, false>(a.grad + c.cb, c.count, lane, x);
    }
    clear_words<R, NW>(lane, wave, sm);   // while the loads are in flight
    if (a.scales_in == nullptr) {
        if (c.full) {
            reduce_minmax<R, WPB, NW, true>(x, c.count, lane, wave, slot, c.seg_lanes, c.rpb, sm, lw);
        } else {
            reduce_minmax<R, WPB, NW, false>(x, c.count, lane, wave, slot, c.seg_lanes, c.rpb, sm, lw);
        }
    }
    if (WPB > 1) __syncthreads();   // every wave of the group arrives here exactly once
    if (!c.active) return;
    if (c.full) {
        encode_minmax_and_pack<R, WPB, NW, true>(a, c.cb, c.count, lane, wave, slot, c.nbc, c.kb_first, x, sm, lw);
    } else {
        encode_minmax_and_pack<R, WPB, NW, false>(a, c.cb, c.count, lane, wave, slot, c.nbc, c.kb_first, x, sm, lw);
    }
}

template <int R, int WPB, int NW>
__global__ __launch_bounds__(64 * NW) void quantize_minmax_wave_kernel(const QuantizeArgs a) {
    __shared__ WaveShared<R, NW> sm;
    __shared__ WaveLows<R, NW> lw;
    quantize_minmax_wave_block<R, WPB, NW>(a, blockIdx.x, sm, lw);
}

// Several layer tensors in one launch, as quantize_tensors_wave_kernel maps them.
template <int R, int WPB, int NW>
__global__ __launch_bounds__(64 * NW) void quantize_minmax_tensors_wave_kernel(const BatchQuantizeArgs ba) {
    __shared__ WaveShared<R, NW> sm;
    __shared__ WaveLows<R, NW> lw;
    uint32_t lo = 0, hi = ba.count;          // tile_start[lo] <= blockIdx.x < tile_start[hi]
    while (hi - lo > 1u) {
        const uint32_t mid = (lo + hi) >> 1;
        if (blockIdx.x >= ba.tile_start[mid]) lo = mid; else hi = mid;
    }
    QuantizeArgs a = ba.common;
    a.grad = ba.t[lo].grad;
    a.n = ba.t[lo].n;
    a.packed = ba.t[lo].packed;
    a.scales = ba.t[lo].scales;
    a.scales_in = ba.t[lo].scales_in;
    quantize_minmax_wave_block<R, WPB, NW>(a, blockIdx.x - ba.tile_start[lo], sm, lw);
}

// The measured choice of (R, WPB, NW) per bucket size (100 M elements, every width): buckets up to 1024
// elements live inside one wave that holds 2048 elements (R = 8); buckets of 2048 .. 8192 span waves of
// 1024 elements each, 4 or 8 to a workgroup; 16384 spans 8 waves of 2048.
template <bool EIGHT, class F>
auto with_wave_shape_w(uint32_t bucket, uint32_t bits, F f) {
    using std::integral_constant;
    using free = integral_constant<int, 8>;   // no cap on the waves per SIMD
    using early = std::true_type;              // random numbers drawn before the range reduction's barrier
    using late = std::false_type;
    // at 8 bits the packed chunk of a 2048-element wave is at its largest; 1024 elements per wave are as fast or faster there
    if constexpr (EIGHT) {
        if (bucket == 512u || bucket == 1024u) {
            return f(integral_constant<int, 4>{}, integral_constant<int, 1>{}, integral_constant<int, 4>{}, free{}, late{});
        }
    }
    // Where a barrier lines eight waves of a workgroup up (buckets 8192 and 16384), drawing before it
    // fills the time the waves would otherwise spend waiting for each other: 1-4 us faster at every
    // width; with four waves per workgroup (2048, 4096) it makes no difference (measured, 100 M elements).
    switch (bucket) {
        case 2048: return f(integral_constant<int, 4>{}, integral_constant<int, 2>{}, integral_constant<int, 4>{}, free{}, late{});
        case 4096: return f(integral_constant<int, 4>{}, integral_constant<int, 4>{}, integral_constant<int, 4>{}, free{}, late{});
        case 8192: return f(integral_constant<int, 4>{}, integral_constant<int, 8>{}, integral_constant<int, 8>{}, free{}, early{});
        case 16384: return f(integral_constant<int, 8>{}, integral_constant<int, 8>{}, integral_constant<int, 8>{}, free{}, early{});
        default:   // 32 .. 1024
            if constexpr (!EIGHT) {
                if (bits <= 3u) return f(integral_constant<int, 8>{}, integral_constant<int, 1>{}, integral_constant<int, 4>{}, free{}, late{});
            }
            return f(integral_constant<int, 8>{}, integral_constant<int, 1>{}, integral_constant<int, 4>{}, integral_constant<int, 5>{}, late{});
    }
}
template <class F>
auto with_wave_shape(uint32_t bucket, uint32_t bits, F f) {
    return bits == 8u ? with_wave_shape_w<true>(bucket, bits, f) : with_wave_shape_w<false>(bucket, bits, f);
}

template <int R, int WPB, int NW, int OCC, bool HOIST>
hipError_t launch_wave(const QuantizeArgs& a, hipStream_t stream) {
    const uint64_t per_group = (uint64_t)NW * 256u * R;
    const uint64_t groups = (a.n + per_group - 1) / per_group;
    if (groups > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL((quantize_wave_kernel<R, WPB, NW, OCC, HOIST>), dim3((uint32_t)groups), dim3(64 * NW), 0, stream, a);
    return hipGetLastError();
}

}  // namespace

// True when the wave-local kernel covers this call: every power-of-two bucket (any 4-byte alignment:
// the 128-bit accesses only need dword alignment).
bool quantize_wave_supported(const QuantizeArgs& a) { return a.bucket_shift >= 5; }

// elements per workgroup of the wave-local kernel at this bucket size
uint32_t quantize_wave_block_elems(uint32_t bucket, uint32_t bits) {
    return with_wave_shape(bucket, bits, [](auto r, auto, auto nw, auto, auto) { return (uint32_t)(decltype(nw)::value * 256 * decltype(r)::value); });
}

hipError_t launch_quantize_tensors_wave(const BatchQuantizeArgs& a, uint32_t blocks, hipStream_t stream) {
    return with_wave_shape(a.common.bucket, a.common.bits, [&](auto r, auto wpb, auto nw, auto occ, auto hoist) {
        constexpr int R = decltype(r)::value, WPB = decltype(wpb)::value, NW = decltype(nw)::value, OCC = decltype(occ)::value;
        constexpr bool HOIST = decltype(hoist)::value;
        hipLaunchKernelGGL((quantize_tensors_wave_kernel<R, WPB, NW, OCC, HOIST>), dim3(blocks), dim3(64 * NW), 0, stream, a);
        return hipGetLastError();
    });
}

hipError_t launch_quantize_wave(const QuantizeArgs& a, hipStream_t stream) {
    return with_wave_shape(a.bucket, a.bits, [&](auto r, auto wpb, auto nw, auto occ, auto hoist) {
        return launch_wave<decltype(r)::value, decltype(wpb)::value, decltype(nw)::value, decltype(occ)::value,
                           decltype(hoist)::value>(a, stream);
    });
}

// Buckets of a whole number of cells that are not powers of two, up to 4064 elements, with the max-abs
// range or given scales.
bool quantize_cells_supported(const QuantizeArgs& a) {
    return a.bucket_shift < 0 && a.bucket <= 4096u && (a.scales_in != nullptr || a.scale_mode == MQG_SCALE_MAXABS);
}
// the batched call: layers without given scales compute them, so the range must be max-abs
bool quantize_tensors_cells_supported(const BatchQuantizeArgs& a) {
    return a.common.bucket_shift < 0 && a.common.bucket <= 4096u && a.common.scale_mode == MQG_SCALE_MAXABS;
}

// Four waves per workgroup unless a larger workgroup's NW * 64 cells are filled at least a tenth better
// by whole buckets: measured at 100 M elements, buckets of 2752 elements (67 % of four waves, 84 % of
// eight) gain 7 us per launch from the larger workgroup, buckets of 1504 (92 % of four, 98 % of six) lose
// 4 us with six.  Up to seven waves: for no admissible bucket do eight fill a tenth better than seven
// or fewer.
static CellGeometry cell_geometry(uint32_t bucket, uint32_t* nw_out) {
    const uint32_t bc = bucket >> 5;
    uint32_t nw = 4u;
    for (uint32_t w = 5u; w <= 7u; ++w) {
        // used fractions (w * 64 / bc) * bc / (w * 64), compared by cross-multiplication
        if (((w * 64u) / bc) * bc * nw * 10u > ((nw * 64u) / bc) * bc * w * 11u) nw = w;
    }
    CellGeometry g;
    g.bucket_cells = bc;
    g.tile_buckets = (nw * 64u) / bc;
    g.tile_cells = g.tile_buckets * bc;
    g.cells_per_wave = (g.tile_cells + nw - 1u) / nw;
    g.magic = (65536u + bc - 1u) / bc;
    *nw_out = nw;
    return g;
}

uint32_t quantize_cells_tile_elems(uint32_t bucket) {
    uint32_t nw;
    return cell_geometry(bucket, &nw).tile_cells * 32u;
}

// Five waves per SIMD instead of six pay where a wave writes much or places many codes across word
// boundaries (measured at 100 M elements: buckets 96 and 480 from 3 bits on by 2-4 us, 1504 at 7 and 8 bits)
static bool cells_cap_occupancy(uint32_t bits, uint32_t bucket) { return bits >= (bucket < 1024u ? 3u : 7u); }

template <int NW>
static hipError_t launch_cells_nw(const QuantizeArgs& a, const CellGeometry& g, uint32_t tiles, hipStream_t stream) {
    if (cells_cap_occupancy(a.bits, a.bucket)) hipLaunchKernelGGL((quantize_cells_kernel<NW, 5, false>), dim3(tiles), dim3(64 * NW), 0, stream, a, g);
    else hipLaunchKernelGGL((quantize_cells_kernel<NW, 8, false>), dim3(tiles), dim3(64 * NW), 0, stream, a, g);
    return hipGetLastError();
}
template <int NW>
static hipError_t launch_tensors_cells_nw(const BatchQuantizeArgs& a, const CellGeometry& g, uint32_t tiles, hipStream_t stream) {
    if (cells_cap_occupancy(a.common.bits, a.common.bucket)) hipLaunchKernelGGL((quantize_tensors_cells_kernel<NW, 5, false>), dim3(tiles), dim3(64 * NW), 0, stream, a, g);
    else hipLaunchKernelGGL((quantize_tensors_cells_kernel<NW, 8, false>), dim3(tiles), dim3(64 * NW), 0, stream, a, g);
    return hipGetLastError();
}

// `tiles` counts tiles of quantize_cells_tile_elems(bucket) elements over all layers
hipError_t launch_quantize_tensors_cells(const BatchQuantizeArgs& a, uint32_t tiles, hipStream_t stream) {
    uint32_t nw;
    const CellGeometry g = cell_geometry(a.common.bucket, &nw);
    switch (nw) {
        case 5: return launch_tensors_cells_nw<5>(a, g, tiles, stream);
        case 6: return launch_tensors_cells_nw<6>(a, g, tiles, stream);
        case 7: return launch_tensors_cells_nw<7>(a, g, tiles, stream);
        default: return launch_tensors_cells_nw<4>(a, g, tiles, stream);
    }
}

hipError_t launch_quantize_cells(const QuantizeArgs& a, hipStream_t stream) {
    uint32_t nw;
    const CellGeometry g = cell_geometry(a.bucket, &nw);
    const uint64_t tile_elems = (uint64_t)g.tile_cells * 32u;
    const uint64_t tiles = (a.n + tile_elems - 1) / tile_elems;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    switch (nw) {
        case 5: return launch_cells_nw<5>(a, g, (uint32_t)tiles, stream);
        case 6: return launch_cells_nw<6>(a, g, (uint32_t)tiles, stream);
        case 7: return launch_cells_nw<7>(a, g, (uint32_t)tiles, stream);
        default: return launch_cells_nw<4>(a, g, (uint32_t)tiles, stream);
    }
}

// The [min, max] encoder takes the same shapes (a given whole-tensor range needs no bucket at all and
// runs the barrier-free shape).
bool quantize_minmax_wave_supported(const QuantizeArgs& a) { return a.bucket_shift >= 5; }

template <int R, int WPB, int NW>
hipError_t launch_minmax_wave(const QuantizeArgs& a, hipStream_t stream) {
    const uint64_t per_group = (uint64_t)NW * 256u * R;
    const uint64_t groups = (a.n + per_group - 1) / per_group;
    if (groups > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)groups), block(64 * NW);
    hipLaunchKernelGGL((quantize_minmax_wave_kernel<R, WPB, NW>), grid, block, 0, stream, a);
    return hipGetLastError();
}

// With no random numbers to draw this encoder is light on the vector ALU, and 1024 elements per wave
// beat 2048 at every bucket size up to 1024 (63-65 us against 70 us at 1 bit, 100 M elements).
// Calls f(R, WPB, NW) with the shape as compile-time constants.
template <class F>
auto with_minmax_wave_shape(uint32_t bucket, F f) {
    using std::integral_constant;
    switch (bucket) {
        case 2048: return f(integral_constant<int, 4>{}, integral_constant<int, 2>{}, integral_constant<int, 4>{});
        case 4096: return f(integral_constant<int, 4>{}, integral_constant<int, 4>{}, integral_constant<int, 4>{});
        case 8192: return f(integral_constant<int, 4>{}, integral_constant<int, 8>{}, integral_constant<int, 8>{});
        case 16384: return f(integral_constant<int, 8>{}, integral_constant<int, 8>{}, integral_constant<int, 8>{});
        default: return f(integral_constant<int, 4>{}, integral_constant<int, 1>{}, integral_constant<int, 4>{});   // 32 .. 1024
    }
}

hipError_t launch_quantize_minmax_wave(const QuantizeArgs& a, hipStream_t stream) {
    return with_minmax_wave_shape(a.bucket, [&](auto r, auto wpb, auto nw) {
        return launch_minmax_wave<decltype(r)::value, decltype(wpb)::value, decltype(nw)::value>(a, stream);
    });
}

// elements per workgroup of the wave-local [min, max] encoder at this bucket size
uint32_t quantize_minmax_wave_block_elems(uint32_t bucket) {
    return with_minmax_wave_shape(bucket, [](auto r, auto, auto nw) { return (uint32_t)(decltype(nw)::value * 256 * decltype(r)::value); });
}

hipError_t launch_quantize_minmax_tensors_wave(const BatchQuantizeArgs& a, uint32_t blocks, hipStream_t stream) {
    return with_minmax_wave_shape(a.common.bucket, [&](auto r, auto wpb, auto nw) {
        constexpr int R = decltype(r)::value, WPB = decltype(wpb)::value, NW = decltype(nw)::value;
        hipLaunchKernelGGL((quantize_minmax_tensors_wave_kernel<R, WPB, NW>), dim3(blocks), dim3(64 * NW), 0, stream, a);
        return hipGetLastError();
    });
}

// The re-quantizing server step takes the wave-local kernel for power-of-two buckets of 128 elements
// and more.
bool requantize_wave_supported(const RequantArgs& ra) { return ra.q.bucket_shift >= 7; }

hipError_t launch_requantize_wave(const RequantArgs& ra, hipStream_t stream) {
    switch (ra.q.bucket) {   // measured choices (100 M elements, W = 8)
        case 2048: return launch_requant_wave<4, 2, 4>(ra, stream);
        case 4096: return launch_requant_wave<4, 4, 4>(ra, stream);
        case 8192: return launch_requant_wave<4, 8, 8>(ra, stream);
        case 16384: return launch_requant_wave<8, 8, 8>(ra, stream);   // workgroups of 16 waves are slower
        case 1024: return launch_requant_wave<4, 1, 4>(ra, stream);      // the bucket is the wave's chunk
        case 512: return launch_requant_wave<4, 1, 4, 2>(ra, stream);
        case 256: return launch_requant_wave<4, 1, 4, 1>(ra, stream);
        case 128: return launch_requant_wave<4, 1, 4, 0>(ra, stream);
        default: return hipErrorInvalidValue;   // requantize_wave_supported() admits none other
    }
}

}  // namespace mqg
