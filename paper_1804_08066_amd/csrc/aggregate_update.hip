// Server side of MQGrad's hot path on gfx950, fused into one pass over the parameters:
// De-quantize every worker's packed gradient, average over the W workers, apply the SGD step
// (Algorithm 1: ReceiveQGThenSendQG takes the mean over the P workers; WorkerIterate's last line
// is w <- w - eta g).
//
//   a5  unpack + de-quantize   v_w = (2 c_w - L) * (s_w / L)
//   a6  aggregate              acc = sum_w v_w     (worker order, one fma per worker)
//   a7  update                 p <- fma(-(lr/W), acc, p)
//
// Work decomposition.  A workgroup of 256 lanes owns a tile of 1024*R consecutive parameters
// (R float4 per lane, coalesced 128-bit loads and stores).  The 4 codes of a lane's quad are the
// 4*bits stream bits that start at bit 4*bits*quad: inside one 32-bit word when bits divides 32,
// spilling into the next word otherwise (and that word is the next lane's first word).  Each lane
// fetches its first word of every worker with one aligned dword load -- adjacent lanes read the same
// or adjacent words, so a wave's request is one contiguous run of 32*bits bytes -- and all loads of
// a chunk of 8 workers are issued before any is consumed.  Parameters are touched once and move with
// the non-temporal hint; so do the code words from 4 bits on (decode::codes_read_once).  The
// de-quantized gradient never exists in HBM.
//
// The per-bucket steps d = s_w / L (one IEEE division per bucket and worker) are shared in one of
// two ways.  Buckets that are multiples of 128 elements: a wave's row of 256 parameters touches
// at most two buckets, so lane w divides worker w's scale(s) of the row and the worker loop reads
// them back with v_readlane -- no LDS, no barrier.  Any other bucket size: a table in LDS, one
// barrier.

#include "decode.h"
#include "kernels.h"
#include "tile_io.h"

#include <type_traits>

namespace mqg {
namespace {

constexpr int kChunk = 8;   // workers whose code loads are in flight together
// float4 per lane in the wave-local kernel (2048 parameters per workgroup); four spilled registers at the
// eight waves per SIMD the kernel needs and ran 2-4 times slower
constexpr int kRowsR = 2;

using namespace tile_io;

// acc <- acc / W with one IEEE fp32 division per element; for a power of two, multiplying by 1/W is
// the same correctly rounded scaling in one operation
template <int R>
__device__ __forceinline__ void scale_to_mean(float4 (&acc)[R], uint32_t W) {
    const float Wf = (float)W;
    if ((W & (W - 1u)) == 0u) {
        const float inv = 1.0f / Wf;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            acc[j].x = acc[j].x * inv;
            acc[j].y = acc[j].y * inv;
            acc[j].z = acc[j].z * inv;
            acc[j].w = acc[j].w * inv;
        }
    } else {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            acc[j].x = acc[j].x / Wf;
            acc[j].y = acc[j].y / Wf;
            acc[j].z = acc[j].z / Wf;
            acc[j].w = acc[j].w / Wf;
        }
    }
}

using decode::accumulate_quad;
using decode::readlane_f32;
// ---- buckets that are multiples of 128: bucket steps live in the wave ---------------------------
// NBR = buckets a 256-element row can touch: 1 when the bucket is a multiple of 256, else 2.
// MEAN: a.params is an output that receives acc / W (the mean gradient) instead of being updated.
// Eight waves per SIMD (64 vector registers): the kernel hides memory latency with occupancy, and seven
// waves cost more than the few spared instructions bring (measured at 100 M parameters).
// LUT > 0: widths 1, 2, 3 decode through the multiplier table in LDS (LUT = the width).
template <int R, int NBR, bool STRADDLE, bool ONCE, int WIDTH, bool MEAN = false, int LUT = 0>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void aggregate_update_rows_kernel(const AggregateArgs a) {
    constexpr uint32_t TILE = 1024u * R;
    __shared__ __attribute__((aligned(16))) float lut[LUT > 0 ? decode::kLutFloats : 1];
    const uint32_t tid = threadIdx.x;
    if (LUT > 0) decode::build_pair_lut(lut, a.bits, tid);
    const uint32_t lane = tid & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6));   // uniform: what follows from it is scalar work
    const uint64_t tile_base = (uint64_t)blockIdx.x * TILE;
    const uint64_t left = a.n - tile_base;
    const uint32_t tile_count = left < TILE ? (uint32_t)left : TILE;
    const bool full = tile_count == TILE;
    float* __restrict__ p = a.params + tile_base;

    // lane w holds worker w's scale pointer (one vector load from the kernel-argument table)
    const float* my_scales = a.scales[lane < a.W ? lane : 0u];

    float4 x[R];
    if (MEAN) {
#pragma unroll
        for (int j = 0; j < R; ++j) x[j] = make_float4(-0.0f, -0.0f, -0.0f, -0.0f);   // fma(1, v, -0) = v for every v
    } else {
        load_params<R>(p, tile_count, full, x);
    }

    const uint32_t b = a.bits;
    const decode::Centred cd = decode::centred(b);
    const float Lf = (float)((1u << b) - 1u);
    const decode::CodeWindows<R> cw = decode::code_windows<R, kThreads>(a.n, tile_base, b, tid);
    decode::CodeRegs<R, kChunk> c;
    decode::fetch_codes<R, kChunk, ONCE>(a.packed, a.W, 0u, cw, c);

    // bucket steps of this wave's rows: lane w divides worker w's scale(s)
    const uint64_t nb_total = (a.n + a.bucket - 1u) / a.bucket;
    const uint64_t kb0 = tile_base / a.bucket;
    const uint32_t first_off = (uint32_t)(tile_base - kb0 * a.bucket);
    float d[R][NBR];
    bool second[R];   // this lane's quad lies in the row's second bucket
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t row_off = first_off + 1024u * j + 256u * wave;   // row start relative to bucket kb0
        const uint32_t kr = a.bucket_shift >= 0 ? (row_off >> a.bucket_shift) : (row_off / a.bucket);
        const uint32_t in_bucket = row_off - kr * a.bucket;
        second[j] = (NBR > 1) && (in_bucket + 4u * lane >= a.bucket);
#pragma unroll
        for (int i = 0; i < NBR; ++i) {
            uint64_t kb = kb0 + kr + i;
            if (kb >= nb_total) kb = nb_total - 1u;   // row (or its second bucket) past the end
            d[j][i] = my_scales[kb] / Lf;             // IEEE-correct fp32 division
        }
    }

    float4 acc[R];
#pragma unroll
    for (int j = 0; j < R; ++j) acc[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (LUT > 0) __syncthreads();   // the table is complete (every wave arrives here exactly once)

    for (uint32_t w0 = 0; w0 < a.W; w0 += kChunk) {
        if (w0 > 0) decode::fetch_codes<R, kChunk, ONCE>(a.packed, a.W, w0, cw, c);
#pragma unroll
        for (int t = 0; t < kChunk; ++t) {
            if (w0 + t < a.W) {
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    float dw = readlane_f32(d[j][0], w0 + t);
                    if (NBR > 1) dw = second[j] ? readlane_f32(d[j][NBR - 1], w0 + t) : dw;
                    if (LUT > 0) {
                        decode::accumulate_quad_lut<LUT>(c.lo[t][j], cw.sh, lut, dw, acc[j]);
                    } else {
                        decode::accumulate_quad_w<STRADDLE, WIDTH>(c.lo[t][j], cw.sh, cd, dw, acc[j]);
                    }
                }
            }
        }
    }
    if (MEAN) {
        scale_to_mean<R>(acc, a.W);
        update_params<R>(p, tile_count, full, 1.0f, x, acc);
    } else {
        update_params<R>(p, tile_count, full, a.neg_c, x, acc);
    }
}

// ---- any other bucket size: bucket steps shared through LDS -------------------------------------
constexpr int kLdsR = 2;
constexpr uint32_t kLdsTile = 1024u * kLdsR;
constexpr uint32_t kMaxBuckets = kLdsTile / 32u + 1u;   // buckets a tile can touch

// One tile of kLdsTile parameters of one tensor.  packed / scales: tables of W device pointers
// (in kernel-argument memory).  raw != nullptr: an uncompressed layer -- the W pointers are fp32
// gradients that are summed in worker order instead of decoded.
// MEAN: `params` is an output that receives acc / W (the mean gradient) instead of being updated.
template <bool STRADDLE, bool ONCE, bool MEAN = false>
__device__ __forceinline__ void aggregate_tile_lds(const uint32_t* const* packed, const float* const* scales,
                                                   const float* const* raw, uint32_t W, uint64_t n, uint32_t b,
                                                   uint32_t bucket, int bucket_shift, float neg_c,
                                                   float* __restrict__ params, uint64_t tile_base, float* s_step) {
    constexpr int R = kLdsR;
    const uint32_t tid = threadIdx.x;
    const uint64_t left = n - tile_base;
    const uint32_t tile_count = left < kLdsTile ? (uint32_t)left : kLdsTile;
    const bool full = tile_count == kLdsTile;
    float* __restrict__ p = params + tile_base;

    float4 x[R];
    if (MEAN) {
#pragma unroll
        for (int j = 0; j < R; ++j) x[j] = make_float4(-0.0f, -0.0f, -0.0f, -0.0f);   // fma(1, v, -0) = v for every v
    } else {
        load_params<R>(p, tile_count, full, x);
    }
    float4 acc[R];
#pragma unroll
    for (int j = 0; j < R; ++j) acc[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);

    if (raw != nullptr) {
        tile_io::accumulate_raw<R>(raw, W, tile_base, tile_count, full, acc);   // uncompressed layer: plain fp32 sum in worker order
        update_params<R>(p, tile_count, full, neg_c, x, acc);
        return;
    }

    const decode::Centred cd = decode::centred(b);
    const float Lf = (float)((1u << b) - 1u);
    const decode::CodeWindows<R> cw = decode::code_windows<R, kThreads>(n, tile_base, b, tid);
    decode::CodeRegs<R, kChunk> c;
    decode::fetch_codes<R, kChunk, ONCE>(packed, W, 0u, cw, c);   // in flight while the bucket steps are computed

    const uint64_t kb0 = tile_base / bucket;
    const uint32_t nbt = (uint32_t)((tile_base + tile_count - 1u) / bucket - kb0) + 1u;   // <= kMaxBuckets
    const uint32_t first_off = (uint32_t)(tile_base - kb0 * bucket);
    uint32_t bl[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t eo = 4u * (j * kThreads + tid) + first_off;
        bl[j] = bucket_shift >= 0 ? (eo >> bucket_shift) : (eo / bucket);
        if (bl[j] >= nbt) bl[j] = nbt - 1u;   // quads past the end: any valid slot
    }
    if (tid < nbt) {
        for (uint32_t w0 = 0; w0 < W; w0 += kChunk) {
            float sv[kChunk];
#pragma unroll
            for (int t = 0; t < kChunk; ++t) {
                const uint32_t w = (w0 + t < W) ? w0 + t : W - 1u;
                sv[t] = scales[w][kb0 + tid];
            }
#pragma unroll
            for (int t = 0; t < kChunk; ++t) {
                if (w0 + t < W) s_step[(w0 + t) * nbt + tid] = sv[t] / Lf;   // IEEE-correct fp32 division
            }
        }
    }
    __syncthreads();

    for (uint32_t w0 = 0; w0 < W; w0 += kChunk) {
        if (w0 > 0) decode::fetch_codes<R, kChunk, ONCE>(packed, W, w0, cw, c);
#pragma unroll
        for (int t = 0; t < kChunk; ++t) {
            if (w0 + t < W) {
                const float* __restrict__ dw = s_step + (w0 + t) * nbt;
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    accumulate_quad<STRADDLE>(c.lo[t][j], cw.sh, cd, dw[bl[j]], acc[j]);
                }
            }
        }
    }
    if (MEAN) {
        // mean = acc / W with one IEEE fp32 division per element; x = -0, so the store's fma(1, mean, -0) is mean
        scale_to_mean<R>(acc, W);
        update_params<R>(p, tile_count, full, 1.0f, x, acc);
        return;
    }
    update_params<R>(p, tile_count, full, neg_c, x, acc);
}

template <bool STRADDLE, bool ONCE>
__global__ __launch_bounds__(kThreads) void aggregate_update_lds_kernel(const AggregateArgs a) {
    extern __shared__ float s_step[];   // [W][nbt]
    aggregate_tile_lds<STRADDLE, ONCE>(a.packed, a.scales, nullptr, a.W, a.n, a.bits, a.bucket, a.bucket_shift,
                                          a.neg_c, a.params, (uint64_t)blockIdx.x * kLdsTile, s_step);
}

template <bool STRADDLE, bool ONCE>
__global__ __launch_bounds__(kThreads) void aggregate_mean_kernel(const AggregateArgs a) {
    extern __shared__ float s_step[];   // [W][nbt]
    aggregate_tile_lds<STRADDLE, ONCE, true>(a.packed, a.scales, nullptr, a.W, a.n, a.bits, a.bucket,
                                                      a.bucket_shift, 0.0f, a.params, (uint64_t)blockIdx.x * kLdsTile, s_step);
}

// Several tensors of a model in one launch: block -> (tensor, tile) through the prefix table of tile
// counts.  A tensor is either quantized (W packed + W scale pointers) or raw (W fp32 gradients).
template <bool STRADDLE, bool ONCE>
__global__ __launch_bounds__(kThreads) void aggregate_update_tensors_kernel(const BatchAggregateArgs a) {
    extern __shared__ float s_step[];
    uint32_t lo = 0, hi = a.count;           // tile_start[lo] <= blockIdx.x < tile_start[hi]
    while (hi - lo > 1u) {
        const uint32_t mid = (lo + hi) >> 1;
        if (blockIdx.x >= a.tile_start[mid]) lo = mid; else hi = mid;
    }
    const BatchAggregateArgs::Tensor& t = a.t[lo];
    const uint64_t tile_base = (uint64_t)(blockIdx.x - a.tile_start[lo]) * kLdsTile;
    const void* const* ptrs = a.ptrs + t.first_ptr;
    if (t.raw) {
        aggregate_tile_lds<STRADDLE, ONCE>(nullptr, nullptr, reinterpret_cast<const float* const*>(ptrs), a.W, t.n,
                                              a.bits, a.bucket, a.bucket_shift, a.neg_c, t.params, tile_base, s_step);
    } else {
        aggregate_tile_lds<STRADDLE, ONCE>(reinterpret_cast<const uint32_t* const*>(ptrs),
                                              reinterpret_cast<const float* const*>(ptrs + a.W), nullptr, a.W, t.n,
                                              a.bits, a.bucket, a.bucket_shift, a.neg_c, t.params, tile_base, s_step);
    }
}

// Calls f(read_once) with the flag as a compile-time constant.
template <class F>
void with_once(bool once, F f) {
    if (once) f(std::true_type{}); else f(std::false_type{});
}

template <int R, int NBR, bool STRADDLE>
hipError_t launch_rows(const AggregateArgs& a, hipStream_t stream) {
    const uint32_t tile = 1024u * R;
    const uint64_t tiles = (a.n + tile - 1) / tile;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)tiles), block(kThreads);
    // Up to 3 bits the step is bound by vector-ALU issue once there are more than eight workers; there the
    // codes are decoded through the multiplier table in LDS (measured at 100 M parameters, 16 workers: 181,
    // 222, 271 us against 199, 246, 280 us; with eight workers the direct forms are 1-3 % faster).
    // streaming loads of the code words: by the width, or because the caller says they come from memory
    const bool once_now = decode::codes_read_once(a.bits) || a.stream_codes != 0u;
    if (a.W > 8u && a.bits <= 3u) {
        with_once(once_now, [&](auto once) {
            constexpr bool ONCE = decltype(once)::value;
            if (a.bits == 1u) hipLaunchKernelGGL((aggregate_update_rows_kernel<R, NBR, false, ONCE, 0, false, 1>), grid, block, 0, stream, a);
            if (a.bits == 2u) hipLaunchKernelGGL((aggregate_update_rows_kernel<R, NBR, false, ONCE, 0, false, 2>), grid, block, 0, stream, a);
            if (a.bits == 3u) hipLaunchKernelGGL((aggregate_update_rows_kernel<R, NBR, true, ONCE, 0, false, 3>), grid, block, 0, stream, a);
        });
        return hipGetLastError();
    }
    if (a.bits == 1u || a.bits == 8u) {   // three-operation decodes; neither width straddles words
        if (a.bits == 1u) {
            with_once(once_now, [&](auto once) {
                hipLaunchKernelGGL((aggregate_update_rows_kernel<R, NBR, false, decltype(once)::value, 1>), grid, block, 0, stream, a);
            });
        } else {
            hipLaunchKernelGGL((aggregate_update_rows_kernel<R, NBR, false, true, 8>), grid, block, 0, stream, a);
        }
        return hipGetLastError();
    }
    with_once(once_now, [&](auto once) {
        hipLaunchKernelGGL((aggregate_update_rows_kernel<R, NBR, STRADDLE, decltype(once)::value, 0>),
                           grid, block, 0, stream, a);
    });
    return hipGetLastError();
}

template <bool STRADDLE>
hipError_t launch_lds(const AggregateArgs& a, hipStream_t stream) {
    const uint64_t tiles = (a.n + kLdsTile - 1) / kLdsTile;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)tiles), block(kThreads);
    const size_t lds = sizeof(float) * a.W * kMaxBuckets;
    with_once(decode::codes_read_once(a.bits) || a.stream_codes != 0u, [&](auto once) {
        hipLaunchKernelGGL((aggregate_update_lds_kernel<STRADDLE, decltype(once)::value>),
                           grid, block, lds, stream, a);
    });
    return hipGetLastError();
}

template <bool STRADDLE>
hipError_t launch_tensors(const BatchAggregateArgs& a, uint32_t tiles, hipStream_t stream) {
    const dim3 grid(tiles), block(kThreads);
    const size_t lds = sizeof(float) * a.W * kMaxBuckets;
    with_once(decode::codes_read_once(a.bits), [&](auto once) {
        hipLaunchKernelGGL((aggregate_update_tensors_kernel<STRADDLE, decltype(once)::value>),
                           grid, block, lds, stream, a);
    });
    return hipGetLastError();
}

template <int R, int NBR, bool STRADDLE>
hipError_t launch_mean_rows(const AggregateArgs& a, hipStream_t stream) {
    const uint32_t tile = 1024u * R;
    const uint64_t tiles = (a.n + tile - 1) / tile;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)tiles), block(kThreads);
    with_once(decode::codes_read_once(a.bits), [&](auto once) {
        hipLaunchKernelGGL((aggregate_update_rows_kernel<R, NBR, STRADDLE, decltype(once)::value, 0, true>),
                           grid, block, 0, stream, a);
    });
    return hipGetLastError();
}

template <bool STRADDLE>
hipError_t launch_mean_s(const AggregateArgs& a, hipStream_t stream) {
    const uint64_t tiles = (a.n + kLdsTile - 1) / kLdsTile;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)tiles), block(kThreads);
    const size_t lds = sizeof(float) * a.W * kMaxBuckets;
    with_once(decode::codes_read_once(a.bits), [&](auto once) {
        hipLaunchKernelGGL((aggregate_mean_kernel<STRADDLE, decltype(once)::value>),
                           grid, block, lds, stream, a);
    });
    return hipGetLastError();
}

}  // namespace

// a.params: the output (n floats); a.neg_c unused
hipError_t launch_aggregate_mean(const AggregateArgs& a, hipStream_t stream) {
    if (a.n == 0) return hipSuccess;
    constexpr int R = kRowsR;
    const bool straddle = (32u % a.bits) != 0u;
    if (a.bucket % 256u == 0u) {
        return straddle ? launch_mean_rows<R, 1, true>(a, stream) : launch_mean_rows<R, 1, false>(a, stream);
    }
    if (a.bucket % 128u == 0u) {
        return straddle ? launch_mean_rows<R, 2, true>(a, stream) : launch_mean_rows<R, 2, false>(a, stream);
    }
    return straddle ? launch_mean_s<true>(a, stream) : launch_mean_s<false>(a, stream);
}

uint32_t aggregate_batch_tile() { return kLdsTile; }

hipError_t launch_aggregate_tensors(const BatchAggregateArgs& a, uint32_t tiles, hipStream_t stream) {
    if (tiles == 0) return hipSuccess;
    const bool straddle = (32u % a.bits) != 0u;
    return straddle ? launch_tensors<true>(a, tiles, stream) : launch_tensors<false>(a, tiles, stream);
}

hipError_t launch_aggregate(const AggregateArgs& a, hipStream_t stream) {
    if (a.n == 0) return hipSuccess;
    constexpr int R = kRowsR;
    const bool straddle = (32u % a.bits) != 0u;   // widths 3, 5, 6, 7
    if (a.bucket % 256u == 0u) {
        return straddle ? launch_rows<R, 1, true>(a, stream) : launch_rows<R, 1, false>(a, stream);
    }
    if (a.bucket % 128u == 0u) {
        return straddle ? launch_rows<R, 2, true>(a, stream) : launch_rows<R, 2, false>(a, stream);
    }
    return straddle ? launch_lds<true>(a, stream) : launch_lds<false>(a, stream);
}

}  // namespace mqg
