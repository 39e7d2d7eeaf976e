// Quantize(g, K) of Algorithm 1 on gfx950, workgroup-cooperative variant: the range-linear K-bit
// encode of the Section 3.2 footnote in ONE pass over its input.  This kernel takes every bucket
// size (any multiple of 32) and both scale modes; power-of-two buckets go to the wave-local kernel in
// quantize_wave.hip instead.
//
//   a1  per-bucket range  s = max |g|            (DPP max over 8-lane cells, LDS max per bucket)
//   a2  position on the 2^K-level grid           u = clamp(fma(g, (L/2)/s, L/2), 0, L)
//   a3  stochastic rounding with Philox4x32-10   c = floor(u) + [(h + 1/2)/65536 < frac(u)]
//   a4  dense little-endian bit packing          LDS-staged, whole words stored coalesced
//
// The values to quantize come from a "source":
//   GradSource    the worker's fp32 gradient (WorkerIterate: Quantize(g, K));
//   DecodeSource  the sum over the W workers' de-quantized gradients, decoded on the fly from their
//                 packed streams (ReceiveQGThenSendQG: the server quantizes the mean and sends it
//                 back).  The division by W is applied to the stored bucket range, not to every
//                 element: the grid of the sum over [-S, S] is the grid of the mean over [-S/W, S/W].
//
// Work decomposition.  A workgroup of 256 lanes owns one tile = a whole number of buckets, at most
// CAP = 1024*R elements, and keeps it in registers (R float4 per lane) between the range
// reduction and the rounding, so each input byte is read from HBM exactly once.  Row j of a
// tile is the 1024 consecutive elements that the 256 lanes hold with one float4 each; 8
// consecutive lanes hold a 32-element "cell", which never straddles a bucket (buckets are
// multiples of 32) and packs into exactly `bits` words.
//
// Random numbers.  One Philox call yields 8 16-bit uniforms for 8 consecutive elements, i.e. for
// the quads of an even/odd lane pair.  So that no lane computes a call whose output is thrown
// away, the even lane computes the pair's call for row j and the odd lane the call for row j+1;
// they swap halves with one DPP quad permute per word.

#include "decode.h"
#include "encode.h"
#include "kernels.h"

namespace mqg {
namespace {

using namespace encode;

constexpr int kThreads = 256;

template <int R>
struct Tile {
    static constexpr uint32_t kCap = 1024u * R;             // elements
    static constexpr uint32_t kMaxWords = kCap * 8u / 32u;  // at 8 bits
    static constexpr uint32_t kMaxBuckets = R > 4 ? 1u : 128u;
};

template <int R>
struct Shared {
    uint32_t words[Tile<R>::kMaxWords + 4];   // packed output of the tile
    uint32_t bmax[128];                       // per-bucket range as fp32 bits
    float ainv[128];                          // per-bucket (L/2)/s
    float cellsq[Tile<R>::kCap / 32u];        // per-cell sum of squares (L2 mode only)
};

// bucket (tile-local) of each of the lane's quads
template <int R>
__device__ __forceinline__ void bucket_of_quads(uint32_t bucket, int bucket_shift, uint32_t (&bl)[R]) {
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t el = 4u * (j * kThreads + threadIdx.x);
        bl[j] = (R > 4) ? 0u : (bucket_shift >= 0 ? (el >> bucket_shift) : (el / bucket));
    }
}

// ---- source: the worker's gradient ---------------------------------------------------------------
template <int R>
struct GradSource {
    const float* __restrict__ g;
    float4 v[R];

    // issue the loads of the tile (one HBM pass)
    __device__ __forceinline__ void issue(uint32_t tile_count, bool full) {
        const uint32_t tid = threadIdx.x;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint32_t el = 4u * (j * kThreads + tid);
            if (full || el + 4u <= tile_count) {
                const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f_a4*>(g + el));   // read once: streaming
                v[j] = make_float4(t.x, t.y, t.z, t.w);
            } else {
                v[j].x = (el + 0u < tile_count) ? g[el + 0] : 0.0f;
                v[j].y = (el + 1u < tile_count) ? g[el + 1] : 0.0f;
                v[j].z = (el + 2u < tile_count) ? g[el + 2] : 0.0f;
                v[j].w = 0.0f;   // el + 3 >= tile_count here
            }
        }
    }
    // after the first barrier: hand over the values
    __device__ __forceinline__ void finish(float4 (&x)[R]) {
#pragma unroll
        for (int j = 0; j < R; ++j) x[j] = v[j];
    }
};

// ---- source: sum over workers of their de-quantized gradients -------------------------------------
// CH workers' code words are in flight together; the per-bucket steps s_w / L of every worker go
// through an LDS table [W][buckets of the tile] that is complete after the tile's first barrier.
template <int R, int CH, bool ONCE>
struct DecodeSource {
    const RequantArgs& ra;
    float* s_step;                       // LDS, W * nbt floats
    uint32_t nbt;                        // buckets in the tile
    decode::CodeWindows<R> cw;
    decode::CodeRegs<R, CH> c;

    __device__ __forceinline__ DecodeSource(const RequantArgs& ra_, float* lds) : ra(ra_), s_step(lds), nbt(0) {}

    __device__ __forceinline__ void issue(uint64_t tile_base, uint32_t tile_count) {
        const uint32_t b = ra.q.bits;
        cw = decode::code_windows<R, kThreads>(ra.q.n, tile_base, b, threadIdx.x);
        decode::fetch_codes<R, CH, ONCE>(ra.packed, ra.W, 0u, cw, c);
        nbt = (R > 4) ? 1u : (tile_count + ra.q.bucket - 1u) / ra.q.bucket;
        const uint64_t kb0 = tile_base / ra.q.bucket;
        const float Lf = (float)((1u << b) - 1u);
        for (uint32_t i = threadIdx.x; i < ra.W * nbt; i += kThreads) {
            const uint32_t w = i / nbt, kb = i - w * nbt;
            s_step[i] = ra.scales[w][kb0 + kb] / Lf;   // IEEE-correct fp32 division
        }
    }
    __device__ __forceinline__ void finish(float4 (&x)[R], uint32_t tile_count, bool full) {
        const uint32_t b = ra.q.bits;
        const decode::Centred cd = decode::centred(b);
        const bool straddle = (32u % b) != 0u;
        uint32_t bl[R];
        bucket_of_quads<R>(ra.q.bucket, ra.q.bucket_shift, bl);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (bl[j] >= nbt) bl[j] = nbt - 1u;   // quads past the end: any valid slot
            x[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
        for (uint32_t w0 = 0; w0 < ra.W; w0 += CH) {
            if (w0 > 0) decode::fetch_codes<R, CH, ONCE>(ra.packed, ra.W, w0, cw, c);
#pragma unroll
            for (int t = 0; t < CH; ++t) {
                if (w0 + t < ra.W) {
                    const float* __restrict__ dw = s_step + (w0 + t) * nbt;
#pragma unroll
                    for (int j = 0; j < R; ++j) {
                        if (straddle) {
                            decode::accumulate_quad<true>(c.lo[t][j], cw.sh, cd, dw[bl[j]], x[j]);
                        } else {
                            decode::accumulate_quad<false>(c.lo[t][j], cw.sh, cd, dw[bl[j]], x[j]);
                        }
                    }
                }
            }
        }
        if (!full) {   // elements past the end decode clamped words: they must not reach the range
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const uint32_t el = 4u * (j * kThreads + threadIdx.x);
                if (el + 0u >= tile_count) x[j].x = 0.0f;
                if (el + 1u >= tile_count) x[j].y = 0.0f;
                if (el + 2u >= tile_count) x[j].z = 0.0f;
                if (el + 3u >= tile_count) x[j].w = 0.0f;
            }
        }
    }
};

// ---- the tile, once its values are in registers ----------------------------------------------------
// Enters right after the barrier that follows the clearing of sm.words / sm.bmax.
// range_div: the stored scale is range / range_div (1 for a plain quantize, W for the mean).
template <int R, bool FULL>
__device__ __forceinline__ void quantize_tile(const QuantizeArgs& a, const uint64_t tile_base,
                                              const uint32_t tile_count, const float4 (&x)[R], float range_div,
                                              Shared<R>& sm) {
    const uint32_t tid = threadIdx.x;
    const uint32_t nbt = (R > 4) ? 1u : (tile_count + a.bucket - 1u) / a.bucket;   // buckets in the tile
    const uint64_t kb0 = tile_base / a.bucket;
    const bool compute_scales = a.scales_in == nullptr;
    const bool l2 = compute_scales && a.scale_mode == MQG_SCALE_L2;
    uint32_t bl[R];
    bucket_of_quads<R>(a.bucket, a.bucket_shift, bl);

    // ---- a1: bucket range -------------------------------------------------------------------
    if (compute_scales) {
        // 8-lane cells by DPP, and one lane per cell folds the result into the bucket's LDS slot.
        // Same-address LDS atomics serialize: when a slot would receive more than 32 of them (buckets
        // of 2048 elements and more) the lane's rows of one bucket are folded first and the reduction
        // goes on over the whole wave, which leaves one atomic per wave (and row).
        constexpr bool kOne = R > 4;                                   // the tile is one bucket
        const bool row_in_bucket = kOne || ((a.bucket & 255u) == 0u && a.bucket >= 2048u);   // uniform over the launch
        if (row_in_bucket) {
            uint32_t m[R];   // bit patterns of non-negative floats: integer order = value order
#pragma unroll
            for (int j = 0; j < R; ++j) {
                m[j] = __builtin_bit_cast(uint32_t, fmaxf(fmaxf(fabsf(x[j].x), fabsf(x[j].y)), fmaxf(fabsf(x[j].z), fabsf(x[j].w))));
            }
            if (kOne) {
#pragma unroll
                for (int j = 1; j < R; ++j) m[0] = max(m[0], m[j]);
            }
#pragma unroll
            for (int j = 0; j < (kOne ? 1 : R); ++j) m[j] = cell_max_u32(m[j]);
#pragma unroll
            for (int j = 0; j < (kOne ? 1 : R); ++j) m[j] = wave_max_from_cells_u32(m[j], tid & 63u);
#pragma unroll
            for (int j = 0; j < (kOne ? 1 : R); ++j) {
                const uint32_t row_first = 4u * (j * kThreads + (tid & ~63u));
                if ((tid & 63u) == 0u && (FULL || kOne || row_first < tile_count)) atomicMax(&sm.bmax[bl[j]], m[j]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const uint32_t el = 4u * (j * kThreads + tid);
                const float mf = fmaxf(fmaxf(fabsf(x[j].x), fabsf(x[j].y)), fmaxf(fabsf(x[j].z), fabsf(x[j].w)));
                const uint32_t m = cell_max_u32(__builtin_bit_cast(uint32_t, mf));
                if ((tid & 7u) == 0u && (FULL || el < tile_count)) atomicMax(&sm.bmax[bl[j]], m);
            }
        }
        if (l2) {
            // sum of squares of each 32-element cell, in a fixed order (reproducible)
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const uint32_t ql = j * kThreads + tid;
                float q = (x[j].x * x[j].x + x[j].y * x[j].y) + (x[j].z * x[j].z + x[j].w * x[j].w);
                q += dpp_f32<kDppQuadSwap1>(q);
                q += dpp_f32<kDppQuadSwap2>(q);
                q += dpp_f32<kDppRowHalfMirror>(q);
                if ((tid & 7u) == 0u) sm.cellsq[ql >> 3] = q;   // zero for cells past the end
            }
        }
    }
    __syncthreads();
    if (l2) {
        // one wave per bucket: lanes add the bucket's cell sums (stride 64) in fp64, then a
        // butterfly over the wave; the norm is raised to max|g| if rounding left it below
        const uint32_t cpb = a.bucket >> 5;
        const uint32_t lane = tid & 63u;
        for (uint32_t k = tid >> 6; k < nbt; k += kThreads / 64) {
            double acc = 0.0;
            for (uint32_t c = lane; c < cpb; c += 64u) acc += (double)sm.cellsq[k * cpb + c];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
            if (lane == 0u) {
                const float norm = (float)__builtin_sqrt(acc);
                const float mx = __builtin_bit_cast(float, sm.bmax[k]);
                sm.bmax[k] = __builtin_bit_cast(uint32_t, norm < mx ? mx : norm);
            }
        }
        __syncthreads();
    }

    const float Lf = (float)((1u << a.bits) - 1u);
    const float halfL = 0.5f * Lf;
    if (tid < nbt) {
        float s;
        if (compute_scales) {
            s = __builtin_bit_cast(float, sm.bmax[tid]);
            if (!(s >= 0x1p-96f)) s = 0.0f;
        } else {
            s = a.scales_in[kb0 + tid];
        }
        a.scales[kb0 + tid] = (range_div == 1.0f) ? s : s / range_div;
        // IEEE-correct fp32 division, once per bucket; kept times 2^16 (exact) for the fixed-point rounding
        sm.ainv[tid] = (s > 0.0f) ? (halfL / s) * 65536.0f : 0.0f;
    }
    __syncthreads();

    // ---- a2..a4: grid position, stochastic rounding, packing --------------------------------
    const uint32_t odd = tid & 1u;
    const uint64_t group0 = (a.elem_base + tile_base) >> 3;   // both multiples of 8
    const uint32_t b = a.bits;
    const FixedGrid fg = fixed_grid(b);
    const uint32_t cell_bit = 4u * b * (tid & 7u);            // this lane's bit offset in its cell
    const uint32_t sh = cell_bit & 31u;
    const uint32_t word_in_cell = cell_bit >> 5;
    const bool straddle = sh + 4u * b > 32u;

#pragma unroll
    for (int jp = 0; jp < R; jp += 2) {
        // the even lane draws for row jp, the odd lane for row jp + 1
        const uint32_t my_row = jp + odd;
        const uint64_t grp = group0 + (uint64_t)((my_row * kThreads + tid) >> 1);
        uint32_t o[4];
        philox4x32_10<true>((uint32_t)grp, (uint32_t)(grp >> 32), a.iteration, a.worker, a.key0, a.key1, o);   // complemented words
        // the swaps run with every lane active; the selects keep the half each lane needs
        const uint32_t p0 = dpp_u32<kDppQuadSwap1>(o[0]), p1 = dpp_u32<kDppQuadSwap1>(o[1]);
        const uint32_t p2 = dpp_u32<kDppQuadSwap1>(o[2]), p3 = dpp_u32<kDppQuadSwap1>(o[3]);
        const uint32_t rw[2][2] = {{odd ? p2 : o[0], odd ? p3 : o[1]},    // row jp: the even lane's call
                                   {odd ? o[2] : p0, odd ? o[3] : p1}};   // row jp+1: the odd lane's call
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int j = jp + t;
            const uint32_t ql = j * kThreads + tid;
            const uint32_t el = 4u * ql;
            const float ainv = sm.ainv[bl[j]];
            uint32_t t0 = round_code_hi(x[j].x, ainv, fg, rw[t][0] & 0xFFFFu);
            uint32_t t1 = round_code_hi(x[j].y, ainv, fg, rw[t][0] >> 16);
            uint32_t t2 = round_code_hi(x[j].z, ainv, fg, rw[t][1] & 0xFFFFu);
            uint32_t t3 = round_code_hi(x[j].w, ainv, fg, rw[t][1] >> 16);
            if (!FULL) {   // elements past the end contribute zero bits
                if (el + 0u >= tile_count) t0 = 0u;
                if (el + 1u >= tile_count) t1 = 0u;
                if (el + 2u >= tile_count) t2 = 0u;
                if (el + 3u >= tile_count) t3 = 0u;
            }
            const uint32_t v = pack_quad_hi(t0, t1, t2, t3, b, 2u * b, 3u * b);
            if (FULL || el < tile_count) {
                const uint32_t w0 = (ql >> 3) * b + word_in_cell;
                atomicOr(&sm.words[w0], v << sh);
                if (straddle) atomicOr(&sm.words[w0 + 1u], v >> (32u - sh));
            }
        }
    }
    __syncthreads();

    // ---- store whole words, coalesced -------------------------------------------------------
    const uint32_t nwords = (tile_count * b + 31u) >> 5;
    uint32_t* __restrict__ out = a.packed + (tile_base >> 5) * b;
    for (uint32_t i = tid; i < nwords; i += kThreads) __builtin_nontemporal_store(sm.words[i], out + i);
}

template <int R>
__device__ __forceinline__ void clear_shared(Shared<R>& sm, uint32_t tile_count, uint32_t bits) {
    const uint32_t nwords = (tile_count * bits + 31u) >> 5;
    for (uint32_t i = threadIdx.x; i < nwords; i += kThreads) sm.words[i] = 0u;
    if (threadIdx.x < 128u) sm.bmax[threadIdx.x] = 0u;
}

template <int R>
__global__ __launch_bounds__(kThreads) void quantize_pack_kernel(const QuantizeArgs a, const uint32_t tile_elems) {
    __shared__ Shared<R> sm;
    const uint64_t tile_base = (uint64_t)blockIdx.x * tile_elems;
    const uint64_t left = a.n - tile_base;
    const uint32_t tile_count = left < tile_elems ? (uint32_t)left : tile_elems;
    const bool full = tile_count == Tile<R>::kCap;

    GradSource<R> src;
    src.g = a.grad + tile_base;
    src.issue(tile_count, full);
    clear_shared<R>(sm, tile_count, a.bits);   // while the loads are in flight
    __syncthreads();
    float4 x[R];
    src.finish(x);
    if (full) {
        quantize_tile<R, true>(a, tile_base, tile_count, x, 1.0f, sm);
    } else {
        quantize_tile<R, false>(a, tile_base, tile_count, x, 1.0f, sm);
    }
}

template <int R, int CH, bool ONCE>
__global__ __launch_bounds__(kThreads) void requantize_pack_kernel(const RequantArgs ra, const uint32_t tile_elems) {
    __shared__ Shared<R> sm;
    extern __shared__ float s_step[];   // [W][buckets of the tile]
    const QuantizeArgs& a = ra.q;
    const uint64_t tile_base = (uint64_t)blockIdx.x * tile_elems;
    const uint64_t left = a.n - tile_base;
    const uint32_t tile_count = left < tile_elems ? (uint32_t)left : tile_elems;
    const bool full = tile_count == Tile<R>::kCap;

    DecodeSource<R, CH, ONCE> src(ra, s_step);
    src.issue(tile_base, tile_count);
    clear_shared<R>(sm, tile_count, a.bits);
    __syncthreads();                      // step table complete, staging clear
    float4 x[R];
    src.finish(x, tile_count, full);      // x = sum over workers of the de-quantized gradients
    const float Wf = (float)ra.W;
    if (full) {
        quantize_tile<R, true>(a, tile_base, tile_count, x, Wf, sm);
    } else {
        quantize_tile<R, false>(a, tile_base, tile_count, x, Wf, sm);
    }
}

// Several layer tensors of one worker in one launch: block -> (tensor, tile) through the prefix table.
template <int R>
__global__ __launch_bounds__(kThreads) void quantize_tensors_kernel(const BatchQuantizeArgs ba) {
    __shared__ Shared<R> sm;
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
    const uint64_t tile_base = (uint64_t)(blockIdx.x - ba.tile_start[lo]) * ba.tile_elems;
    const uint64_t left = a.n - tile_base;
    const uint32_t tile_count = left < ba.tile_elems ? (uint32_t)left : ba.tile_elems;
    const bool full = tile_count == Tile<R>::kCap;

    GradSource<R> src;
    src.g = a.grad + tile_base;
    src.issue(tile_count, full);
    clear_shared<R>(sm, tile_count, a.bits);
    __syncthreads();
    float4 x[R];
    src.finish(x);
    if (full) {
        quantize_tile<R, true>(a, tile_base, tile_count, x, 1.0f, sm);
    } else {
        quantize_tile<R, false>(a, tile_base, tile_count, x, 1.0f, sm);
    }
}

template <int R>
hipError_t launch_tensors_r(const BatchQuantizeArgs& a, uint32_t tiles, hipStream_t stream) {
    hipLaunchKernelGGL((quantize_tensors_kernel<R>), dim3(tiles), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

template <int R>
hipError_t launch_r(const QuantizeArgs& a, hipStream_t stream) {
    const uint32_t cap = Tile<R>::kCap;
    const uint32_t tile_elems = (cap / a.bucket) * a.bucket;   // whole buckets, >= 1 by choice of R
    const uint64_t tiles = (a.n + tile_elems - 1) / tile_elems;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL((quantize_pack_kernel<R>), dim3((uint32_t)tiles), dim3(kThreads), 0, stream, a, tile_elems);
    return hipGetLastError();
}

template <int R, int CH>
hipError_t launch_requant_r(const RequantArgs& ra, hipStream_t stream) {
    const uint32_t cap = Tile<R>::kCap;
    const uint32_t tile_elems = (cap / ra.q.bucket) * ra.q.bucket;
    const uint64_t tiles = (ra.q.n + tile_elems - 1) / tile_elems;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const size_t lds = sizeof(float) * ra.W * Tile<R>::kMaxBuckets;
    if (decode::codes_read_once(ra.q.bits)) {
        hipLaunchKernelGGL((requantize_pack_kernel<R, CH, true>), dim3((uint32_t)tiles), dim3(kThreads), lds, stream, ra, tile_elems);
    } else {
        hipLaunchKernelGGL((requantize_pack_kernel<R, CH, false>), dim3((uint32_t)tiles), dim3(kThreads), lds, stream, ra, tile_elems);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_quantize(const QuantizeArgs& a, hipStream_t stream) {
    if (a.n == 0) return hipSuccess;
    if (quantize_wave_supported(a)) return launch_quantize_wave(a, stream);
    if (quantize_cells_supported(a)) return launch_quantize_cells(a, stream);
    if (a.bucket <= 4096u) return launch_r<4>(a, stream);
    if (a.bucket <= 8192u) return launch_r<8>(a, stream);
    return launch_r<16>(a, stream);
}

// Power-of-two buckets take the wave-local kernel, like single calls.
static bool batch_takes_wave_kernel(int bucket_shift) { return bucket_shift >= 5; }

uint32_t quantize_batch_tile(const BatchQuantizeArgs& a) {
    const uint32_t bucket = a.common.bucket;
    if (batch_takes_wave_kernel(a.common.bucket_shift)) return quantize_wave_block_elems(bucket, a.common.bits);
    if (quantize_tensors_cells_supported(a)) return quantize_cells_tile_elems(bucket);
    const uint32_t cap = bucket <= 4096u ? Tile<4>::kCap : (bucket <= 8192u ? Tile<8>::kCap : Tile<16>::kCap);
    return (cap / bucket) * bucket;
}

hipError_t launch_quantize_tensors(const BatchQuantizeArgs& a, uint32_t tiles, hipStream_t stream) {
    if (tiles == 0) return hipSuccess;
    if (batch_takes_wave_kernel(a.common.bucket_shift)) return launch_quantize_tensors_wave(a, tiles, stream);
    if (quantize_tensors_cells_supported(a)) return launch_quantize_tensors_cells(a, tiles, stream);
    if (a.common.bucket <= 4096u) return launch_tensors_r<4>(a, tiles, stream);
    if (a.common.bucket <= 8192u) return launch_tensors_r<8>(a, tiles, stream);
    return launch_tensors_r<16>(a, tiles, stream);
}

hipError_t launch_requantize(const RequantArgs& ra, hipStream_t stream) {
    if (ra.q.n == 0) return hipSuccess;
    if (requantize_wave_supported(ra)) return launch_requantize_wave(ra, stream);
    if (ra.q.bucket <= 4096u) return launch_requant_r<4, 8>(ra, stream);
    if (ra.q.bucket <= 8192u) return launch_requant_r<8, 4>(ra, stream);
    return launch_requant_r<16, 2>(ra, stream);
}

}  // namespace mqg
