// The Section 3.2 footnote read literally, on gfx950: a deterministic range-linear encode of a
// gradient to K bits over the [min, max] of each bucket (bucket >= n: one range per tensor, as in the
// paper), the matching server step, and the sum of squares that the "Adaptive" baseline's bit rule
// (Section 4.1) needs.
//
//   encode   mn, mx per bucket;  a = L / (mx - mn);  c = clamp(rint((g - mn) * a), 0, L)
//   decode   value = fma((float)c, (mx - mn) / L, mn)
//   server   acc = sum_w value_w (worker order);  p <- fma(-(lr/W), acc, p)
//
// No random numbers.  Work decomposition as in the stochastic quantizer's workgroup-cooperative
// kernel: a workgroup owns one tile of whole buckets (four float4 per lane, 256 to 1024 lanes, read
// from HBM once), ranges go through LDS with order-preserving integer keys, codes are packed through
// LDS and whole words are stored coalesced.

#include <mutex>

#include "decode.h"
#include "encode.h"
#include "kernels.h"
#include "tile_io.h"

namespace mqg {
namespace {

using namespace encode;
using tile_io::kThreads;

constexpr int kChunk = 8;   // workers whose code loads are in flight together
// The whole-tensor reductions end with one atomic per workgroup on one address; those serialize at
// about 5 ns each and every workgroup arrives at the end together, so the workgroups are few and large:
// 512 of 512 lanes (8 waves per SIMD) read as fast as 2048 of 256 and end 7 us earlier at 100 M elements.
constexpr int kSumThreads = 512;
constexpr uint32_t kSumBlocks = 512;

// NT lanes own a tile of at most 4*NT*R elements
template <int R, int NT>
struct Shared {
    static constexpr uint32_t kCap = 4u * NT * R;
    static constexpr bool kOneBucket = kCap > 4096u;   // tiles above 4096 elements are chosen for one large bucket
    uint32_t words[kCap * 8u / 32u + 4];
    uint32_t kmin[128];
    uint32_t kmax[128];
    float mn[128];
    float a[128];
};

// one HBM pass: the tile of the gradient into registers
template <int R, int NT, bool FULL>
__device__ __forceinline__ void load_grad_tile(const float* __restrict__ g, const uint32_t tile_count, float4 (&x)[R]) {
    const uint32_t tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t el = 4u * (j * NT + tid);
        if (FULL || el + 4u <= tile_count) {
            const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f_a4*>(g + el));
            x[j] = make_float4(t.x, t.y, t.z, t.w);
        } else {
            x[j].x = (el + 0u < tile_count) ? g[el + 0] : 0.0f;
            x[j].y = (el + 1u < tile_count) ? g[el + 1] : 0.0f;
            x[j].z = (el + 2u < tile_count) ? g[el + 2] : 0.0f;
            x[j].w = 0.0f;   // el + 3 >= tile_count here
        }
    }
}

template <int R, int NT>
__device__ __forceinline__ void clear_shared(Shared<R, NT>& sm, uint32_t tile_count, uint32_t b) {
    const uint32_t tid = threadIdx.x;
    const uint32_t nwords = (tile_count * b + 31u) >> 5;
    for (uint32_t i = tid; i < nwords; i += NT) sm.words[i] = 0u;
    if (tid < 128u) {
        sm.kmin[tid] = 0xFFFFFFFFu;
        sm.kmax[tid] = 0u;
    }
}

// The tile, once its values are in registers; enters right after the barrier that follows
// clear_shared.  range_div: the stored range is [mn, mx] / range_div (1 for a plain encode, W for the
// server's mean).
// GIVEN: one (min, max) pair for every element, read from a.scales_in (the whole-tensor range found by
// an earlier pass); no range is reduced and none is stored.
template <int R, int NT, bool FULL, bool GIVEN = false>
__device__ __forceinline__ void encode_minmax_tile(const QuantizeArgs& a, const uint64_t tile_base,
                                                   const uint32_t tile_count, const float4 (&x)[R],
                                                   const float range_div, Shared<R, NT>& sm) {
    const uint32_t tid = threadIdx.x;
    const float inf = __builtin_inff();
    const uint32_t b = a.bits;
    const uint32_t nwords = (tile_count * b + 31u) >> 5;

    const uint32_t nbt = (GIVEN || Shared<R, NT>::kOneBucket) ? 1u : (tile_count + a.bucket - 1u) / a.bucket;   // buckets in the tile
    const uint64_t kb0 = GIVEN ? 0u : tile_base / a.bucket;
    uint32_t bl[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t el = 4u * (j * NT + tid);
        bl[j] = (GIVEN || Shared<R, NT>::kOneBucket) ? 0u : (a.bucket_shift >= 0 ? (el >> a.bucket_shift) : (el / a.bucket));
    }

    // ---- bucket range: 8-lane cells by DPP; whole waves when a wave's row lies in one bucket -------
    // (every lane of a cell, or of a wave, then holds the same value, and one lane folds it into the
    // bucket's LDS slot: few atomics per slot, since same-address LDS atomics serialize)
    constexpr bool kOne = Shared<R, NT>::kOneBucket;
    const uint32_t lane = tid & 63u;
    const bool row_in_bucket = kOne || (a.bucket & 255u) == 0u;   // uniform over the launch
    if (!GIVEN) {
    float lo[R], hi[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t el = 4u * (j * NT + tid);
        if (FULL) {
            lo[j] = fminf(fminf(x[j].x, x[j].y), fminf(x[j].z, x[j].w));
            hi[j] = fmaxf(fmaxf(x[j].x, x[j].y), fmaxf(x[j].z, x[j].w));
        } else {   // elements past the end take no part
            const bool v0 = el + 0u < tile_count, v1 = el + 1u < tile_count;
            const bool v2 = el + 2u < tile_count, v3 = el + 3u < tile_count;
            lo[j] = fminf(fminf(v0 ? x[j].x : inf, v1 ? x[j].y : inf), fminf(v2 ? x[j].z : inf, v3 ? x[j].w : inf));
            hi[j] = fmaxf(fmaxf(v0 ? x[j].x : -inf, v1 ? x[j].y : -inf), fmaxf(v2 ? x[j].z : -inf, v3 ? x[j].w : -inf));
        }
    }
    if (kOne) {   // the tile is one bucket: fold the lane's rows first
#pragma unroll
        for (int j = 1; j < R; ++j) {
            lo[0] = fminf(lo[0], lo[j]);
            hi[0] = fmaxf(hi[0], hi[j]);
        }
    }
    // across lanes on order-preserving integer keys, stage by stage over the rows
    uint32_t kl[R], kh[R];
#pragma unroll
    for (int j = 0; j < (kOne ? 1 : R); ++j) {
        kl[j] = cell_min_u32(order_key(lo[j]));
        kh[j] = cell_max_u32(order_key(hi[j]));
    }
    if (row_in_bucket) {
#pragma unroll
        for (int j = 0; j < (kOne ? 1 : R); ++j) {
            kl[j] = wave_min_from_cells_u32(kl[j], lane);
            kh[j] = wave_max_from_cells_u32(kh[j], lane);
        }
#pragma unroll
        for (int j = 0; j < (kOne ? 1 : R); ++j) {
            const uint32_t row_first = 4u * (j * NT + (tid & ~63u));   // first element of the wave's row
            if (lane == 0u && (FULL || kOne || row_first < tile_count)) {
                atomicMin(&sm.kmin[bl[j]], kl[j]);
                atomicMax(&sm.kmax[bl[j]], kh[j]);
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint32_t el = 4u * (j * NT + tid);
            if ((tid & 7u) == 0u && (FULL || el < tile_count)) {
                atomicMin(&sm.kmin[bl[j]], kl[j]);
                atomicMax(&sm.kmax[bl[j]], kh[j]);
            }
        }
    }
    }
    __syncthreads();

    const float Lf = (float)((1u << b) - 1u);
    if (tid < nbt) {
        float mn, mx;
        if (GIVEN) {
            mn = a.scales_in[0];
            mx = a.scales_in[1];
        } else {
            mn = key_value(sm.kmin[tid]);
            mx = key_value(sm.kmax[tid]);
            if (mn == 0.0f) mn = 0.0f;   // a zero bound is stored as +0
            if (mx == 0.0f) mx = 0.0f;
            a.scales[2u * (kb0 + tid)] = (range_div == 1.0f) ? mn : mn / range_div;
            a.scales[2u * (kb0 + tid) + 1u] = (range_div == 1.0f) ? mx : mx / range_div;
        }
        const float r = mx - mn;
        sm.mn[tid] = mn;
        sm.a[tid] = (r >= 0x1p-96f) ? Lf / r : 0.0f;   // IEEE-correct fp32 division, once per bucket
    }
    __syncthreads();

    // ---- nearest level, packing -----------------------------------------------------------------
    const uint32_t cell_bit = 4u * b * (tid & 7u);            // this lane's bit offset in its 32-element cell
    const uint32_t sh = cell_bit & 31u;
    const uint32_t word_in_cell = cell_bit >> 5;
    const bool straddle = sh + 4u * b > 32u;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t ql = j * NT + tid;
        const uint32_t el = 4u * ql;
        const float mn = sm.mn[bl[j]], ai = sm.a[bl[j]];
        // fmaxf drops a NaN position to 0; positions are integers after rint
        uint32_t k0 = (uint32_t)fminf(fmaxf(__builtin_rintf((x[j].x - mn) * ai), 0.0f), Lf);
        uint32_t k1 = (uint32_t)fminf(fmaxf(__builtin_rintf((x[j].y - mn) * ai), 0.0f), Lf);
        uint32_t k2 = (uint32_t)fminf(fmaxf(__builtin_rintf((x[j].z - mn) * ai), 0.0f), Lf);
        uint32_t k3 = (uint32_t)fminf(fmaxf(__builtin_rintf((x[j].w - mn) * ai), 0.0f), Lf);
        if (!FULL) {   // elements past the end contribute zero bits
            if (el + 0u >= tile_count) k0 = 0u;
            if (el + 1u >= tile_count) k1 = 0u;
            if (el + 2u >= tile_count) k2 = 0u;
            if (el + 3u >= tile_count) k3 = 0u;
        }
        const uint32_t v = (((((k3 << b) | k2) << b) | k1) << b) | k0;
        if (FULL || el < tile_count) {
            const uint32_t w0 = (ql >> 3) * b + word_in_cell;
            atomicOr(&sm.words[w0], v << sh);
            if (straddle) atomicOr(&sm.words[w0 + 1u], v >> (32u - sh));
        }
    }
    __syncthreads();

    uint32_t* __restrict__ out = a.packed + (tile_base >> 5) * b;
    for (uint32_t i = tid; i < nwords; i += NT) __builtin_nontemporal_store(sm.words[i], out + i);
}

// Bucket sizes that are not powers of two (the others take the wave-local kernel in quantize_wave.hip).
template <int R, int NT>
__device__ __forceinline__ void quantize_minmax_tile(const QuantizeArgs& a, const uint32_t tile, const uint32_t tile_elems,
                                                     Shared<R, NT>& sm) {
    const uint64_t tile_base = (uint64_t)tile * tile_elems;
    const uint64_t left = a.n - tile_base;
    const uint32_t tile_count = left < tile_elems ? (uint32_t)left : tile_elems;
    float4 x[R];
    if (tile_count == Shared<R, NT>::kCap) {
        load_grad_tile<R, NT, true>(a.grad + tile_base, tile_count, x);
        clear_shared<R, NT>(sm, tile_count, a.bits);   // while the loads are in flight
        __syncthreads();
        encode_minmax_tile<R, NT, true>(a, tile_base, tile_count, x, 1.0f, sm);
    } else {
        load_grad_tile<R, NT, false>(a.grad + tile_base, tile_count, x);
        clear_shared<R, NT>(sm, tile_count, a.bits);
        __syncthreads();
        encode_minmax_tile<R, NT, false>(a, tile_base, tile_count, x, 1.0f, sm);
    }
}

template <int R, int NT>
__global__ __launch_bounds__(NT) void quantize_minmax_kernel(const QuantizeArgs a, const uint32_t tile_elems) {
    __shared__ Shared<R, NT> sm;
    quantize_minmax_tile<R, NT>(a, blockIdx.x, tile_elems, sm);
}

// Several layer tensors in one launch: workgroup -> (tensor, tile of the tensor) through the prefix
// table of tile counts.
template <int R, int NT>
__global__ __launch_bounds__(NT) void quantize_minmax_tensors_kernel(const BatchQuantizeArgs ba) {
    __shared__ Shared<R, NT> sm;
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
    quantize_minmax_tile<R, NT>(a, blockIdx.x - ba.tile_start[lo], ba.tile_elems, sm);
}

// The server's re-encoding step of the full exchange (ReceiveQGThenSendQG): the tile's values are the
// sum over the W workers' de-quantized gradients, decoded from their streams in worker order; the
// stored range is divided by W.  (step, min) of every worker's buckets of the tile sit in an LDS table.
template <int NT, bool STRADDLE, bool ONCE>
__global__ __launch_bounds__(NT) void requantize_minmax_kernel(const RequantArgs ra, const uint32_t tile_elems) {
    constexpr int R = 4;
    constexpr int CH = 8;   // workers whose code loads are in flight together
    __shared__ Shared<R, NT> sm;
    extern __shared__ float2 s_tab[];   // [W][buckets of the tile]
    const QuantizeArgs& a = ra.q;
    const uint32_t tid = threadIdx.x;
    const uint64_t tile_base = (uint64_t)blockIdx.x * tile_elems;
    const uint64_t left = a.n - tile_base;
    const uint32_t tile_count = left < tile_elems ? (uint32_t)left : tile_elems;
    const bool full = tile_count == Shared<R, NT>::kCap;
    const uint32_t b = a.bits;
    const float Lf = (float)((1u << b) - 1u);

    const decode::CodeWindows<R> cw = decode::code_windows<R, NT>(a.n, tile_base, b, tid);
    decode::CodeRegs<R, CH> c;
    decode::fetch_codes<R, CH, ONCE>(ra.packed, ra.W, 0u, cw, c);   // in flight while the table is filled
    const uint32_t nbt = Shared<R, NT>::kOneBucket ? 1u : (tile_count + a.bucket - 1u) / a.bucket;
    const uint64_t kb0 = tile_base / a.bucket;
    for (uint32_t i = tid; i < ra.W * nbt; i += NT) {
        const uint32_t w = i / nbt, kb = i - w * nbt;
        const float2 rg = reinterpret_cast<const float2*>(ra.scales[w])[kb0 + kb];   // (min, max)
        s_tab[i] = make_float2((rg.y - rg.x) / Lf, rg.x);                            // IEEE-correct fp32 division
    }
    clear_shared<R, NT>(sm, tile_count, b);
    __syncthreads();

    uint32_t bl[R];
    float4 x[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t el = 4u * (j * NT + tid);
        bl[j] = Shared<R, NT>::kOneBucket ? 0u : (a.bucket_shift >= 0 ? (el >> a.bucket_shift) : (el / a.bucket));
        if (bl[j] >= nbt) bl[j] = nbt - 1u;   // quads past the end: any valid slot
        x[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
    for (uint32_t w0 = 0; w0 < ra.W; w0 += CH) {
        if (w0 > 0) decode::fetch_codes<R, CH, ONCE>(ra.packed, ra.W, w0, cw, c);
#pragma unroll
        for (int t = 0; t < CH; ++t) {
            if (w0 + t < ra.W) {
                const float2* __restrict__ tw = s_tab + (w0 + t) * nbt;
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    const float2 sl = tw[bl[j]];
                    decode::accumulate_quad_minmax<STRADDLE>(c.lo[t][j], cw.sh, b, sl.x, sl.y, x[j]);
                }
            }
        }
    }
    const float Wf = (float)ra.W;
    if (full) {
        encode_minmax_tile<R, NT, true>(a, tile_base, tile_count, x, Wf, sm);
    } else {
        encode_minmax_tile<R, NT, false>(a, tile_base, tile_count, x, Wf, sm);   // ignores elements past the end
    }
}

// ---- the same with ONE range for the whole tensor, as the paper encodes -----------------------------
// The range of the sum is not known until every element has been decoded, so the step takes two passes
// over the W code streams (the fp32 sum still never exists in memory: (2 W + 1) * bits / 8 bytes per
// element in all): pass 1 decodes and folds the tile's min / max into two integer keys (exact and order
// independent; a workgroup first looks whether its values can move a key at all, since same-address
// atomics serialize); pass 2 decodes again and encodes over that range.
// Every worker has one (min, max) pair; s_tab[w] = (step, min) of worker w.
template <int NT, bool STRADDLE, bool ONCE>
__device__ __forceinline__ void decode_sum_tile_tensor(const RequantArgs& ra, const uint64_t tile_base, float2* s_tab,
                                                       float4 (&x)[4]) {
    constexpr int R = 4;
    constexpr int CH = 8;
    const uint32_t tid = threadIdx.x;
    const uint32_t b = ra.q.bits;
    const float Lf = (float)((1u << b) - 1u);
    const decode::CodeWindows<R> cw = decode::code_windows<R, NT>(ra.q.n, tile_base, b, tid);
    decode::CodeRegs<R, CH> c;
    decode::fetch_codes<R, CH, ONCE>(ra.packed, ra.W, 0u, cw, c);   // in flight while the table is filled
    if (tid < ra.W) {
        const float2 rg = *reinterpret_cast<const float2*>(ra.scales[tid]);   // (min, max) of worker tid
        s_tab[tid] = make_float2((rg.y - rg.x) / Lf, rg.x);                   // IEEE-correct fp32 division
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < R; ++j) x[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (uint32_t w0 = 0; w0 < ra.W; w0 += CH) {
        if (w0 > 0) decode::fetch_codes<R, CH, ONCE>(ra.packed, ra.W, w0, cw, c);
#pragma unroll
        for (int t = 0; t < CH; ++t) {
            if (w0 + t < ra.W) {
                const float2 sl = s_tab[w0 + t];
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    decode::accumulate_quad_minmax<STRADDLE>(c.lo[t][j], cw.sh, b, sl.x, sl.y, x[j]);
                }
            }
        }
    }
}

template <int NT, bool STRADDLE, bool ONCE>
__global__ __launch_bounds__(NT) void sum_range_minmax_tensor_kernel(const RequantArgs ra, uint32_t* keys) {
    constexpr int R = 4;
    constexpr uint32_t kCap = 4u * NT * R;
    __shared__ float2 s_tab[MQG_MAX_WORKERS];
    __shared__ uint32_t s_lo[NT / 64], s_hi[NT / 64];
    const uint32_t tid = threadIdx.x;
    const uint64_t tile_base = (uint64_t)blockIdx.x * kCap;
    const uint64_t left = ra.q.n - tile_base;
    const uint32_t tile_count = left < kCap ? (uint32_t)left : kCap;
    float4 x[R];
    decode_sum_tile_tensor<NT, STRADDLE, ONCE>(ra, tile_base, s_tab, x);
    const float inf = __builtin_inff();
    float lo = inf, hi = -inf;
#pragma unroll
    for (int j = 0; j < R; ++j) {   // elements past the end take no part
        const uint32_t el = 4u * (j * NT + tid);
        if (el + 0u < tile_count) { lo = fminf(lo, x[j].x); hi = fmaxf(hi, x[j].x); }
        if (el + 1u < tile_count) { lo = fminf(lo, x[j].y); hi = fmaxf(hi, x[j].y); }
        if (el + 2u < tile_count) { lo = fminf(lo, x[j].z); hi = fmaxf(hi, x[j].z); }
        if (el + 3u < tile_count) { lo = fminf(lo, x[j].w); hi = fmaxf(hi, x[j].w); }
    }
    uint32_t kl = wave_min_from_cells_u32(cell_min_u32(order_key(lo)), tid & 63u);
    uint32_t kh = wave_max_from_cells_u32(cell_max_u32(order_key(hi)), tid & 63u);
    if ((tid & 63u) == 0u) {
        s_lo[tid >> 6] = kl;
        s_hi[tid >> 6] = kh;
    }
    __syncthreads();
    if (tid == 0u) {
#pragma unroll
        for (int w = 1; w < NT / 64; ++w) {
            kl = min(kl, s_lo[w]);
            kh = max(kh, s_hi[w]);
        }
        // the keys only ever move one way, so a stale read can cause a needless atomic but never a wrong skip
        if (kl < __atomic_load_n(&keys[0], __ATOMIC_RELAXED)) atomicMin(&keys[0], kl);
        if (kh > __atomic_load_n(&keys[1], __ATOMIC_RELAXED)) atomicMax(&keys[1], kh);
    }
}

template <int NT, bool STRADDLE, bool ONCE>
__global__ __launch_bounds__(NT) void requantize_minmax_tensor_kernel(const RequantArgs ra) {
    constexpr int R = 4;
    constexpr uint32_t kCap = Shared<R, NT>::kCap;
    __shared__ Shared<R, NT> sm;
    __shared__ float2 s_tab[MQG_MAX_WORKERS];
    const uint64_t tile_base = (uint64_t)blockIdx.x * kCap;
    const uint64_t left = ra.q.n - tile_base;
    const uint32_t tile_count = left < kCap ? (uint32_t)left : kCap;
    clear_shared<R, NT>(sm, tile_count, ra.q.bits);
    float4 x[R];
    decode_sum_tile_tensor<NT, STRADDLE, ONCE>(ra, tile_base, s_tab, x);   // its barrier also covers clear_shared
    if (tile_count == kCap) {
        encode_minmax_tile<R, NT, true, true>(ra.q, tile_base, tile_count, x, 1.0f, sm);
    } else {
        encode_minmax_tile<R, NT, false, true>(ra.q, tile_base, tile_count, x, 1.0f, sm);
    }
}

// range[0..1] <- range[0..1] / W: the grid of the mean is the grid of the sum scaled by 1 / W
__global__ void range_divide_kernel(float* range, float Wf) {
    range[0] = range[0] / Wf;
    range[1] = range[1] / Wf;
}

// ---- server step --------------------------------------------------------------------------------
constexpr int kAggR = 2;
constexpr uint32_t kAggTile = 1024u * kAggR;
constexpr uint32_t kMaxBuckets = kAggTile / 32u + 1u;   // buckets a tile can touch

// One tile of one tensor.  The fields of `a` that name the tensor (n, params, packed, scales) are not
// read: the tensor comes in through the arguments, so that one launch can serve several.  raw != nullptr:
// an uncompressed layer whose W fp32 gradients are added in worker order instead of decoded.
struct TileTensor {
    const uint32_t* const* packed;
    const float* const* scales;
    const float* const* raw;
    uint64_t n;
    float* params;
};
struct TileCommon {
    uint32_t W, bits, bucket;
    int bucket_shift;
    uint32_t per_tensor;
    float neg_c;
};
template <bool STRADDLE, bool ONCE>
__device__ __forceinline__ void aggregate_minmax_tile(const TileCommon& a, const TileTensor& t, const uint64_t tile_base,
                                                      float2* s_tab) {
    constexpr int R = kAggR;
    const uint32_t tid = threadIdx.x;
    const uint64_t left = t.n - tile_base;
    const uint32_t tile_count = left < kAggTile ? (uint32_t)left : kAggTile;
    const bool full = tile_count == kAggTile;
    float* __restrict__ p = t.params + tile_base;

    float4 x[R];
    tile_io::load_params<R>(p, tile_count, full, x);
    float4 acc[R];
#pragma unroll
    for (int j = 0; j < R; ++j) acc[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (t.raw != nullptr) {
        tile_io::accumulate_raw<R>(t.raw, a.W, tile_base, tile_count, full, acc);
        tile_io::update_params<R>(p, tile_count, full, a.neg_c, x, acc);
        return;
    }

    const uint32_t b = a.bits;
    const float Lf = (float)((1u << b) - 1u);
    const decode::CodeWindows<R> cw = decode::code_windows<R, kThreads>(t.n, tile_base, b, tid);
    decode::CodeRegs<R, kChunk> c;
    decode::fetch_codes<R, kChunk, ONCE>(t.packed, a.W, 0u, cw, c);   // in flight while the table is filled

    const uint64_t kb0 = tile_base / a.bucket;
    const uint32_t nbt = (uint32_t)((tile_base + tile_count - 1u) / a.bucket - kb0) + 1u;   // <= kMaxBuckets
    const uint32_t first_off = (uint32_t)(tile_base - kb0 * a.bucket);
    uint32_t bl[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t eo = 4u * (j * kThreads + tid) + first_off;
        bl[j] = a.bucket_shift >= 0 ? (eo >> a.bucket_shift) : (eo / a.bucket);
        if (bl[j] >= nbt) bl[j] = nbt - 1u;   // quads past the end: any valid slot
    }
    for (uint32_t i = tid; i < a.W * nbt; i += kThreads) {
        const uint32_t w = i / nbt, kb = i - w * nbt;
        const float2 rg = reinterpret_cast<const float2*>(t.scales[w])[a.per_tensor ? 0u : kb0 + kb];   // (min, max)
        s_tab[i] = make_float2((rg.y - rg.x) / Lf, rg.x);                           // IEEE-correct fp32 division
    }
    __syncthreads();

    for (uint32_t w0 = 0; w0 < a.W; w0 += kChunk) {
        if (w0 > 0) decode::fetch_codes<R, kChunk, ONCE>(t.packed, a.W, w0, cw, c);
#pragma unroll
        for (int t = 0; t < kChunk; ++t) {
            if (w0 + t < a.W) {
                const float2* __restrict__ tw = s_tab + (w0 + t) * nbt;
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    const float2 sl = tw[bl[j]];
                    decode::accumulate_quad_minmax<STRADDLE>(c.lo[t][j], cw.sh, b, sl.x, sl.y, acc[j]);
                }
            }
        }
    }
    tile_io::update_params<R>(p, tile_count, full, a.neg_c, x, acc);
}

template <bool STRADDLE, bool ONCE>
__global__ __launch_bounds__(kThreads) void aggregate_update_minmax_kernel(const AggregateArgs a) {
    extern __shared__ float2 s_tab[];   // [W][nbt]: (step, min) of each worker's buckets of the tile
    const TileCommon c = {a.W, a.bits, a.bucket, a.bucket_shift, a.per_tensor, a.neg_c};
    const TileTensor t = {a.packed, a.scales, nullptr, a.n, a.params};
    aggregate_minmax_tile<STRADDLE, ONCE>(c, t, (uint64_t)blockIdx.x * kAggTile, s_tab);
}

// Several tensors of a model in one launch: block -> (tensor, tile) through the prefix table of tile
// counts.  A tensor is either encoded (W packed + W range pointers) or raw (W fp32 gradients).
template <bool STRADDLE, bool ONCE>
__global__ __launch_bounds__(kThreads) void aggregate_update_minmax_tensors_kernel(const BatchAggregateArgs a) {
    extern __shared__ float2 s_tab[];
    uint32_t lo = 0, hi = a.count;           // tile_start[lo] <= blockIdx.x < tile_start[hi]
    while (hi - lo > 1u) {
        const uint32_t mid = (lo + hi) >> 1;
        if (blockIdx.x >= a.tile_start[mid]) lo = mid; else hi = mid;
    }
    const BatchAggregateArgs::Tensor& bt = a.t[lo];
    const void* const* ptrs = a.ptrs + bt.first_ptr;
    const TileCommon c = {a.W, a.bits, a.bucket, a.bucket_shift, a.per_tensor, a.neg_c};
    TileTensor t = {nullptr, nullptr, nullptr, bt.n, bt.params};
    if (bt.raw) {
        t.raw = reinterpret_cast<const float* const*>(ptrs);
    } else {
        t.packed = reinterpret_cast<const uint32_t* const*>(ptrs);
        t.scales = reinterpret_cast<const float* const*>(ptrs + a.W);
    }
    aggregate_minmax_tile<STRADDLE, ONCE>(c, t, (uint64_t)(blockIdx.x - a.tile_start[lo]) * kAggTile, s_tab);
}

// ---- whole-tensor range ---------------------------------------------------------------------------
// The paper encodes a tensor over ONE range.  Three launches on the stream: a one-thread kernel
// primes range[0..1] with the identity keys, the reduction folds every workgroup's min / max into them
// with integer atomics on order-preserving keys (exact and order-independent), a one-thread kernel
// turns the keys back into floats (a zero bound as +0).
__global__ void range_init_kernel(uint32_t* keys) {
    keys[0] = 0xFFFFFFFFu;
    keys[1] = 0u;
}

__global__ void range_finish_kernel(uint32_t* keys) {
    float mn = key_value(keys[0]), mx = key_value(keys[1]);
    if (mn == 0.0f) mn = 0.0f;
    if (mx == 0.0f) mx = 0.0f;
    keys[0] = __builtin_bit_cast(uint32_t, mn);
    keys[1] = __builtin_bit_cast(uint32_t, mx);
}

// The calling workgroup (`block` of `nblocks`) folds its share of g[0..n) into keys[0..1].
__device__ __forceinline__ void block_range(const float* __restrict__ g, const uint64_t n, const uint32_t block,
                                            const uint32_t nblocks, uint32_t* keys, uint32_t* s_lo, uint32_t* s_hi) {
    const uint32_t tid = threadIdx.x;
    const uint64_t gtid = (uint64_t)block * kSumThreads + tid;
    const uint64_t stride = (uint64_t)nblocks * kSumThreads;
    float lo = __builtin_inff(), hi = -__builtin_inff();
    const v4f_a4* __restrict__ g4 = reinterpret_cast<const v4f_a4*>(g);   // 128-bit loads need dword alignment only
    const uint64_t nq = n >> 2;
    const uint64_t pieces = nq / (4u * kSumThreads);   // contiguous 32 KB pieces, four float4 per lane in flight
    for (uint64_t pc = block; pc < pieces; pc += nblocks) {
        const v4f_a4* __restrict__ src = g4 + pc * (4u * kSumThreads) + tid;
        v4f t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = __builtin_nontemporal_load(src + u * kSumThreads);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            lo = fminf(lo, fminf(fminf(t[u].x, t[u].y), fminf(t[u].z, t[u].w)));
            hi = fmaxf(hi, fmaxf(fmaxf(t[u].x, t[u].y), fmaxf(t[u].z, t[u].w)));
        }
    }
    for (uint64_t q = pieces * (4u * kSumThreads) + gtid; q < nq; q += stride) {   // less than one piece is left
        const v4f t = g4[q];
        lo = fminf(lo, fminf(fminf(t.x, t.y), fminf(t.z, t.w)));
        hi = fmaxf(hi, fmaxf(fmaxf(t.x, t.y), fmaxf(t.z, t.w)));
    }
    if (gtid < (n & 3u)) {
        const float v = g[(nq << 2) + gtid];
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
    uint32_t kl = wave_min_from_cells_u32(cell_min_u32(order_key(lo)), tid & 63u);
    uint32_t kh = wave_max_from_cells_u32(cell_max_u32(order_key(hi)), tid & 63u);
    if ((tid & 63u) == 0u) {
        s_lo[tid >> 6] = kl;
        s_hi[tid >> 6] = kh;
    }
    __syncthreads();
    if (tid == 0u) {
#pragma unroll
        for (int w = 1; w < kSumThreads / 64; ++w) {
            kl = min(kl, s_lo[w]);
            kh = max(kh, s_hi[w]);
        }
        // Same-address atomics serialize in L2: look first.  The keys only ever move one way, so a
        // stale read can cause a needless atomic but never a wrong skip.
        if (kl < __atomic_load_n(&keys[0], __ATOMIC_RELAXED)) atomicMin(&keys[0], kl);
        if (kh > __atomic_load_n(&keys[1], __ATOMIC_RELAXED)) atomicMax(&keys[1], kh);
    }
}

__global__ __launch_bounds__(kSumThreads) void tensor_range_kernel(const float* __restrict__ g, const uint64_t n,
                                                                   uint32_t* keys) {
    __shared__ uint32_t s_lo[kSumThreads / 64], s_hi[kSumThreads / 64];
    block_range(g, n, blockIdx.x, gridDim.x, keys, s_lo, s_hi);
}

// The ranges of several tensors: grid (blocks, tensors); thread k of the one-workgroup kernels before
// and after primes / converts the keys of tensor k.  Empty tensors have no range array.
__global__ void range_init_batch_kernel(const TensorRangeBatch b, uint32_t count) {
    if (threadIdx.x < count && b.range[threadIdx.x] != nullptr) {
        uint32_t* keys = reinterpret_cast<uint32_t*>(b.range[threadIdx.x]);
        keys[0] = 0xFFFFFFFFu;
        keys[1] = 0u;
    }
}
__global__ __launch_bounds__(kSumThreads) void tensor_range_batch_kernel(const TensorRangeBatch b) {
    __shared__ uint32_t s_lo[kSumThreads / 64], s_hi[kSumThreads / 64];
    const uint32_t k = blockIdx.y;
    if (b.range[k] == nullptr) return;
    block_range(b.grad[k], b.n[k], blockIdx.x, gridDim.x, reinterpret_cast<uint32_t*>(b.range[k]), s_lo, s_hi);
}
__global__ void range_finish_batch_kernel(const TensorRangeBatch b, uint32_t count) {
    if (threadIdx.x < count && b.range[threadIdx.x] != nullptr) {
        uint32_t* keys = reinterpret_cast<uint32_t*>(b.range[threadIdx.x]);
        float mn = key_value(keys[0]), mx = key_value(keys[1]);
        if (mn == 0.0f) mn = 0.0f;   // a zero bound is stored as +0
        if (mx == 0.0f) mx = 0.0f;
        keys[0] = __builtin_bit_cast(uint32_t, mn);
        keys[1] = __builtin_bit_cast(uint32_t, mx);
    }
}

// ---- sum of squares -------------------------------------------------------------------------------
// Squares of fp32 values are exact in fp64; every lane adds its share in fp64, lanes and waves are
// combined by a butterfly and through LDS.  Two ways to finish: mqg_sum_squares adds one fp64 number
// per workgroup to *out with an atomic (its rounding depends on the order in which the workgroups
// arrive: about 1e-16 relative); the batched form stores one partial sum per workgroup and a second
// kernel adds them in a fixed order, which makes the result reproducible to the bit.

__global__ void clear_f64_kernel(double* out) { *out = 0.0; }

// The calling workgroup's share of sum g[i]^2 (workgroup `block` of `nblocks`); the value is returned
// in thread 0.  The order of every addition is a function of (n, nblocks) only.
__device__ __forceinline__ double block_sum_squares(const float* __restrict__ g, const uint64_t n, const uint32_t block,
                                                    const uint32_t nblocks, double* s_part) {
    const uint32_t tid = threadIdx.x;
    const uint64_t gtid = (uint64_t)block * kSumThreads + tid;
    const uint64_t stride = (uint64_t)nblocks * kSumThreads;
    double acc = 0.0;
    const v4f_a4* __restrict__ g4 = reinterpret_cast<const v4f_a4*>(g);   // 128-bit loads need dword alignment only
    const uint64_t nq = n >> 2;
    // a workgroup reads 32 KB contiguous pieces (four float4 per lane in flight), pieces nblocks apart
    const uint64_t pieces = nq / (4u * kSumThreads);
    for (uint64_t pc = block; pc < pieces; pc += nblocks) {
        const v4f_a4* __restrict__ src = g4 + pc * (4u * kSumThreads) + tid;
        v4f t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = __builtin_nontemporal_load(src + u * kSumThreads);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const double a0 = (double)t[u].x, a1 = (double)t[u].y, a2 = (double)t[u].z, a3 = (double)t[u].w;
            acc += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
        }
    }
    for (uint64_t q = pieces * (4u * kSumThreads) + gtid; q < nq; q += stride) {   // less than one piece is left
        const v4f t = __builtin_nontemporal_load(g4 + q);
        const double a0 = (double)t.x, a1 = (double)t.y, a2 = (double)t.z, a3 = (double)t.w;
        acc += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
    }
    if (gtid < (n & 3u)) {
        const double v = (double)g[(nq << 2) + gtid];
        acc += v * v;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
    if ((tid & 63u) == 0u) s_part[tid >> 6] = acc;
    __syncthreads();
    double t = 0.0;
    if (tid == 0u) {
#pragma unroll
        for (int w = 0; w < kSumThreads / 64; ++w) t += s_part[w];
    }
    return t;
}

__global__ __launch_bounds__(kSumThreads) void sum_squares_kernel(const float* __restrict__ g, const uint64_t n,
                                                                  double* out) {
    __shared__ double s_part[kSumThreads / 64];
    const double t = block_sum_squares(g, n, blockIdx.x, gridDim.x, s_part);
    if (threadIdx.x == 0u) atomicAdd(out, t);
}

// Batched, ordered form.  blockIdx.y = tensor, blockIdx.x = workgroup of the tensor; every workgroup
// stores its partial sum (0 for a workgroup that has nothing to read), nothing is accumulated in memory.
__global__ __launch_bounds__(kSumThreads) void sum_squares_partial_kernel(const SumSquaresBatch b, double* __restrict__ partials) {
    __shared__ double s_part[kSumThreads / 64];
    const uint32_t k = blockIdx.y;
    const double t = block_sum_squares(b.grad[k], b.n[k], blockIdx.x, gridDim.x, s_part);
    if (threadIdx.x == 0u) partials[(uint64_t)k * gridDim.x + blockIdx.x] = t;
}

// One wave per tensor: lane l adds partials l, l + 64, ... in that order, then the butterfly.
__global__ __launch_bounds__(64) void sum_squares_finish_kernel(const double* __restrict__ partials, const uint32_t nblocks,
                                                                double* __restrict__ out) {
    const double* __restrict__ p = partials + (uint64_t)blockIdx.x * nblocks;
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < nblocks; i += 64u) acc += p[i];
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
    if (threadIdx.x == 0u) out[blockIdx.x] = acc;
}

template <int R, int NT>
hipError_t launch_quantize_r(const QuantizeArgs& a, hipStream_t stream) {
    const uint32_t cap = Shared<R, NT>::kCap;
    const uint32_t tile_elems = (cap / a.bucket) * a.bucket;   // whole buckets, >= 1 by choice of R
    const uint64_t tiles = (a.n + tile_elems - 1) / tile_elems;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)tiles), block(NT);
    if (a.scales_in != nullptr) return hipErrorInvalidValue;   // a given range is tiled with a power-of-two bucket
    hipLaunchKernelGGL((quantize_minmax_kernel<R, NT>), grid, block, 0, stream, a, tile_elems);
    return hipGetLastError();
}

template <bool STRADDLE>
hipError_t launch_aggregate_s(const AggregateArgs& a, hipStream_t stream) {
    const uint64_t tiles = (a.n + kAggTile - 1) / kAggTile;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)tiles), block(kThreads);
    const size_t lds = sizeof(float2) * a.W * kMaxBuckets;
    if (decode::codes_read_once(a.bits)) {
        hipLaunchKernelGGL((aggregate_update_minmax_kernel<STRADDLE, true>), grid, block, lds, stream, a);
    } else {
        hipLaunchKernelGGL((aggregate_update_minmax_kernel<STRADDLE, false>), grid, block, lds, stream, a);
    }
    return hipGetLastError();
}

template <int NT>
hipError_t launch_requant_nt(const RequantArgs& ra, hipStream_t stream) {
    const uint32_t cap = Shared<4, NT>::kCap;
    // whole buckets per tile, and at most 4096 table entries (32 KB of LDS)
    uint32_t nb_tile = cap / ra.q.bucket;
    const uint32_t max_nb = 4096u / ra.W;   // >= 64
    if (nb_tile > max_nb) nb_tile = max_nb;
    const uint32_t tile_elems = nb_tile * ra.q.bucket;
    const uint64_t tiles = (ra.q.n + tile_elems - 1) / tile_elems;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)tiles), block(NT);
    const size_t lds = sizeof(float2) * ra.W * nb_tile;
    const bool straddle = (32u % ra.q.bits) != 0u;
    const bool once = decode::codes_read_once(ra.q.bits);
    if (straddle) {
        if (once) hipLaunchKernelGGL((requantize_minmax_kernel<NT, true, true>), grid, block, lds, stream, ra, tile_elems);
        else hipLaunchKernelGGL((requantize_minmax_kernel<NT, true, false>), grid, block, lds, stream, ra, tile_elems);
    } else {
        if (once) hipLaunchKernelGGL((requantize_minmax_kernel<NT, false, true>), grid, block, lds, stream, ra, tile_elems);
        else hipLaunchKernelGGL((requantize_minmax_kernel<NT, false, false>), grid, block, lds, stream, ra, tile_elems);
    }
    return hipGetLastError();
}

}  // namespace

// ra.scales[w]: worker w's (min, max) pairs; ra.q.scales: (min, max) pairs of the mean
hipError_t launch_requantize_minmax(const RequantArgs& ra, hipStream_t stream) {
    if (ra.q.n == 0) return hipSuccess;
    if (ra.q.bucket <= 4096u) return launch_requant_nt<256>(ra, stream);
    if (ra.q.bucket <= 8192u) return launch_requant_nt<512>(ra, stream);
    return launch_requant_nt<1024>(ra, stream);
}

// a.scales: 2 floats (min, max) per bucket; a.scale_mode, key, iteration, worker, elem_base unused
hipError_t launch_quantize_minmax(const QuantizeArgs& a, hipStream_t stream) {
    if (a.n == 0) return hipSuccess;
    if (quantize_minmax_wave_supported(a)) return launch_quantize_minmax_wave(a, stream);   // power-of-two buckets
    // four float4 per lane at every bucket size; larger buckets take larger workgroups
    if (a.bucket <= 4096u) return launch_quantize_r<4, 256>(a, stream);
    if (a.bucket <= 8192u) return launch_quantize_r<4, 512>(a, stream);
    return launch_quantize_r<4, 1024>(a, stream);
}

// The general tile of the batched encoder: R = 4 with the workgroup size that the bucket needs.
uint32_t quantize_minmax_batch_tile(uint32_t bucket, int bucket_shift) {
    if (bucket_shift >= 5) return quantize_minmax_wave_block_elems(bucket);
    const uint32_t cap = bucket <= 4096u ? Shared<4, 256>::kCap : (bucket <= 8192u ? Shared<4, 512>::kCap : Shared<4, 1024>::kCap);
    return (cap / bucket) * bucket;
}

// a.t[i].scales: (min, max) pairs of tensor i's buckets; a.t[i].scales_in: nullptr, or the ONE (min, max)
// pair of tensor i (then nothing is written to scales and the bucket only shapes the launch: it must be
// a power of two)
hipError_t launch_quantize_minmax_tensors(const BatchQuantizeArgs& a, uint32_t tiles, hipStream_t stream) {
    if (tiles == 0) return hipSuccess;
    if (a.common.bucket_shift >= 5) return launch_quantize_minmax_tensors_wave(a, tiles, stream);
    const dim3 grid(tiles);
    if (a.common.bucket <= 4096u) hipLaunchKernelGGL((quantize_minmax_tensors_kernel<4, 256>), grid, dim3(256), 0, stream, a);
    else if (a.common.bucket <= 8192u) hipLaunchKernelGGL((quantize_minmax_tensors_kernel<4, 512>), grid, dim3(512), 0, stream, a);
    else hipLaunchKernelGGL((quantize_minmax_tensors_kernel<4, 1024>), grid, dim3(1024), 0, stream, a);
    return hipGetLastError();
}

// range[k][0..1] <- min, max of tensor k; three launches on the stream
hipError_t launch_tensor_range_batch(const TensorRangeBatch& b, uint32_t count, hipStream_t stream) {
    uint64_t most = 0;
    for (uint32_t k = 0; k < count; ++k) {
        if (b.range[k] != nullptr && b.n[k] > most) most = b.n[k];
    }
    if (most == 0) return hipSuccess;
    uint64_t blocks = ((most >> 2) + kSumThreads - 1) / kSumThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > kSumBlocks) blocks = kSumBlocks;
    hipLaunchKernelGGL(range_init_batch_kernel, dim3(1), dim3(64), 0, stream, b, count);
    hipLaunchKernelGGL(tensor_range_batch_kernel, dim3((uint32_t)blocks, count), dim3(kSumThreads), 0, stream, b);
    hipLaunchKernelGGL(range_finish_batch_kernel, dim3(1), dim3(64), 0, stream, b, count);
    return hipGetLastError();
}

uint32_t aggregate_minmax_batch_tile() { return kAggTile; }

// a.ptrs: per encoded tensor [W packed][W range arrays], per raw tensor [W fp32 gradients]
hipError_t launch_aggregate_minmax_tensors(const BatchAggregateArgs& a, uint32_t tiles, hipStream_t stream) {
    if (tiles == 0) return hipSuccess;
    const dim3 grid(tiles), block(kThreads);
    const size_t lds = sizeof(float2) * a.W * kMaxBuckets;
    const bool straddle = (32u % a.bits) != 0u;
    const bool once = decode::codes_read_once(a.bits);
    if (straddle) {
        if (once) hipLaunchKernelGGL((aggregate_update_minmax_tensors_kernel<true, true>), grid, block, lds, stream, a);
        else hipLaunchKernelGGL((aggregate_update_minmax_tensors_kernel<true, false>), grid, block, lds, stream, a);
    } else {
        if (once) hipLaunchKernelGGL((aggregate_update_minmax_tensors_kernel<false, true>), grid, block, lds, stream, a);
        else hipLaunchKernelGGL((aggregate_update_minmax_tensors_kernel<false, false>), grid, block, lds, stream, a);
    }
    return hipGetLastError();
}

// a.scales[w]: worker w's (min, max) pairs
hipError_t launch_aggregate_minmax(const AggregateArgs& a, hipStream_t stream) {
    if (a.n == 0) return hipSuccess;
    const bool straddle = (32u % a.bits) != 0u;
    return straddle ? launch_aggregate_s<true>(a, stream) : launch_aggregate_s<false>(a, stream);
}

// ra.scales[w]: worker w's one (min, max) pair; ra.q.scales: the (min, max) pair of the mean (2 floats).
// Five launches on the stream: prime the keys, pass 1, keys -> floats, pass 2, divide the range by W.
hipError_t launch_requantize_minmax_tensor(const RequantArgs& ra_in, hipStream_t stream) {
    if (ra_in.q.n == 0) return hipSuccess;
    constexpr int NT = 256;
    constexpr uint32_t kCap = Shared<4, NT>::kCap;
    const uint64_t tiles = (ra_in.q.n + kCap - 1) / kCap;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    RequantArgs ra = ra_in;
    ra.q.scales_in = ra.q.scales;   // pass 2 reads the range of the sum from where pass 1 left it
    uint32_t* keys = reinterpret_cast<uint32_t*>(ra.q.scales);
    const dim3 grid((uint32_t)tiles), block(NT);
    const bool straddle = (32u % ra.q.bits) != 0u;
    const bool once = decode::codes_read_once(ra.q.bits);
    hipLaunchKernelGGL(range_init_kernel, dim3(1), dim3(1), 0, stream, keys);
    if (straddle) {
        if (once) hipLaunchKernelGGL((sum_range_minmax_tensor_kernel<NT, true, true>), grid, block, 0, stream, ra, keys);
        else hipLaunchKernelGGL((sum_range_minmax_tensor_kernel<NT, true, false>), grid, block, 0, stream, ra, keys);
    } else {
        if (once) hipLaunchKernelGGL((sum_range_minmax_tensor_kernel<NT, false, true>), grid, block, 0, stream, ra, keys);
        else hipLaunchKernelGGL((sum_range_minmax_tensor_kernel<NT, false, false>), grid, block, 0, stream, ra, keys);
    }
    hipLaunchKernelGGL(range_finish_kernel, dim3(1), dim3(1), 0, stream, keys);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (straddle) {
        if (once) hipLaunchKernelGGL((requantize_minmax_tensor_kernel<NT, true, true>), grid, block, 0, stream, ra);
        else hipLaunchKernelGGL((requantize_minmax_tensor_kernel<NT, true, false>), grid, block, 0, stream, ra);
    } else {
        if (once) hipLaunchKernelGGL((requantize_minmax_tensor_kernel<NT, false, true>), grid, block, 0, stream, ra);
        else hipLaunchKernelGGL((requantize_minmax_tensor_kernel<NT, false, false>), grid, block, 0, stream, ra);
    }
    hipLaunchKernelGGL(range_divide_kernel, dim3(1), dim3(1), 0, stream, ra.q.scales, (float)ra.W);
    return hipGetLastError();
}

hipError_t launch_tensor_range(const float* grad, uint64_t n, float* range_out, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    uint32_t* keys = reinterpret_cast<uint32_t*>(range_out);
    hipLaunchKernelGGL(range_init_kernel, dim3(1), dim3(1), 0, stream, keys);
    uint64_t blocks = ((n >> 2) + kSumThreads - 1) / kSumThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > kSumBlocks) blocks = kSumBlocks;
    hipLaunchKernelGGL(tensor_range_kernel, dim3((uint32_t)blocks), dim3(kSumThreads), 0, stream, grad, n, keys);
    hipLaunchKernelGGL(range_finish_kernel, dim3(1), dim3(1), 0, stream, keys);
    return hipGetLastError();
}
uint32_t sum_squares_batch_blocks() { return kSumBlocks; }

// partials: count * kSumBlocks doubles of scratch memory; out: count doubles
hipError_t launch_sum_squares_batch(const SumSquaresBatch& b, uint32_t count, double* partials, double* out, hipStream_t stream) {
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(sum_squares_partial_kernel, dim3(kSumBlocks, count), dim3(kSumThreads), 0, stream, b, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sum_squares_finish_kernel, dim3(count), dim3(64), 0, stream, partials, (uint32_t)kSumBlocks, out);
    return hipGetLastError();
}

// ---- the same with the partial sums in memory that the library itself holds ------------------------
// For callers that cannot allocate (code under graph capture, serving loops): a file-scope device array
// takes the place of the workspace.  Every GPU the library runs on holds its own copy of the array, at
// its own address, until the process ends; the array's name is a host-side handle, not a device address,
// so the address is asked for once per device (with that device current) and kept.
constexpr int kMaxDevices = 64;
static __device__ __align__(256) double scratch[kMaxSumTensors * kSumBlocks];   // 256 KB per GPU

static std::mutex g_scratch_mutex;
static double* g_scratch_ptr[kMaxDevices];   // per device; nullptr until first use on that device

static hipError_t static_scratch(double** ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        double* p = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

// No allocation anywhere on this path; the partial sums are all overwritten before they are read, so
// nothing has to be cleared between calls.
hipError_t launch_sum_squares_batch_static(const SumSquaresBatch& b, uint32_t count, double* out, hipStream_t stream) {
    if (count == 0) return hipSuccess;
    if (count > kMaxSumTensors) return hipErrorInvalidValue;
    double* partials = nullptr;
    const hipError_t e = static_scratch(&partials);
    if (e != hipSuccess) return e;
    return launch_sum_squares_batch(b, count, partials, out, stream);
}

hipError_t launch_sum_squares(const float* grad, uint64_t n, double* out, hipStream_t stream) {
    hipLaunchKernelGGL(clear_f64_kernel, dim3(1), dim3(1), 0, stream, out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n == 0) return e;
    uint64_t blocks = ((n >> 2) + kSumThreads - 1) / kSumThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > kSumBlocks) blocks = kSumBlocks;
    hipLaunchKernelGGL(sum_squares_kernel, dim3((uint32_t)blocks), dim3(kSumThreads), 0, stream, grad, n, out);
    return hipGetLastError();
}

}  // namespace mqg
