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
// (R float4 per lane, coalesced).  The code words of the tile (tile*bits/32 words per worker,
// contiguous because tiles start at multiples of 32 elements) are staged through LDS in chunks of
// workers, together with the per-bucket steps s_w/L, so the small code stream is also read with
// full-width coalesced loads and no lane fetches a word twice from memory.  The de-quantized
// gradient never exists in HBM.

#include "kernels.h"

namespace mqg {
namespace {

constexpr int kThreads = 256;
constexpr int kR = 2;                         // float4 per lane
constexpr uint32_t kTile = 1024u * kR;        // parameters per workgroup
constexpr uint32_t kChunk = 8;                // workers staged in LDS at a time
constexpr uint32_t kMaxWords = kTile * 8u / 32u + 2u;   // per worker, at 8 bits, + pad for the straddle read
constexpr uint32_t kMaxBuckets = kTile / 32u + 1u;      // buckets a tile can touch

template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) void aggregate_update_kernel(const AggregateArgs a) {
    __shared__ uint32_t s_words[kChunk][kMaxWords];
    __shared__ float s_step[kChunk][kMaxBuckets];

    const uint32_t tid = threadIdx.x;
    const uint64_t tile_base = (uint64_t)blockIdx.x * kTile;
    const uint64_t left = a.n - tile_base;
    const uint32_t tile_count = left < kTile ? (uint32_t)left : kTile;
    const bool full = tile_count == kTile;
    float* __restrict__ p = a.params + tile_base;

    // ---- parameters of the tile -------------------------------------------------------------
    float4 x[kR];
#pragma unroll
    for (int j = 0; j < kR; ++j) {
        const uint32_t el = 4u * (j * kThreads + tid);
        if (full || el + 4u <= tile_count) {
            if (ALIGNED) {
                x[j] = *reinterpret_cast<const float4*>(p + el);
            } else {
                x[j] = make_float4(p[el], p[el + 1], p[el + 2], p[el + 3]);
            }
        } else {
            x[j].x = (el + 0u < tile_count) ? p[el + 0] : 0.0f;
            x[j].y = (el + 1u < tile_count) ? p[el + 1] : 0.0f;
            x[j].z = (el + 2u < tile_count) ? p[el + 2] : 0.0f;
            x[j].w = 0.0f;
        }
    }

    const uint32_t b = a.bits;
    const uint32_t L = (1u << b) - 1u;
    const float Lf = (float)L;
    const uint32_t nwords = (tile_count * b + 31u) >> 5;
    const uint64_t word_base = (tile_base >> 5) * b;
    const uint64_t kb0 = tile_base / a.bucket;
    const uint32_t nbt = (uint32_t)((tile_base + tile_count - 1u) / a.bucket - kb0) + 1u;
    const uint32_t first_off = (uint32_t)(tile_base - kb0 * a.bucket);   // offset of the tile in its first bucket

    // per-quad constants
    uint32_t bl[kR], wi[kR], sh[kR];
#pragma unroll
    for (int j = 0; j < kR; ++j) {
        const uint32_t ql = j * kThreads + tid;
        const uint32_t eo = 4u * ql + first_off;
        bl[j] = a.bucket_shift >= 0 ? (eo >> a.bucket_shift) : (eo / a.bucket);
        const uint32_t bit = 4u * b * ql;
        wi[j] = bit >> 5;
        sh[j] = bit & 31u;
    }

    float4 acc[kR];
#pragma unroll
    for (int j = 0; j < kR; ++j) acc[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);

    for (uint32_t w0 = 0; w0 < a.W; w0 += kChunk) {
        const uint32_t wc = (a.W - w0 < kChunk) ? (a.W - w0) : kChunk;
        if (w0 > 0) __syncthreads();   // the previous chunk has been consumed
        // ---- stage code words and bucket steps of workers [w0, w0 + wc) ----------------------
        for (uint32_t w = 0; w < wc; ++w) {
            const uint32_t* __restrict__ src = a.packed[w0 + w] + word_base;
            for (uint32_t i = tid; i < nwords; i += kThreads) s_words[w][i] = src[i];
            if (tid < 2u) s_words[w][nwords + tid] = 0u;
        }
        for (uint32_t i = tid; i < wc * nbt; i += kThreads) {
            const uint32_t w = i / nbt, kb = i - w * nbt;
            s_step[w][kb] = a.scales[w0 + w][kb0 + kb] / Lf;   // IEEE-correct fp32 division
        }
        __syncthreads();

        // ---- a5, a6: unpack, de-quantize, accumulate in worker order ------------------------
        for (uint32_t w = 0; w < wc; ++w) {
#pragma unroll
            for (int j = 0; j < kR; ++j) {
                if (bl[j] >= nbt) continue;   // quad entirely past the end of the vector
                const float d = s_step[w][bl[j]];
                const uint32_t lo = s_words[w][wi[j]];
                const uint32_t hi = s_words[w][wi[j] + 1u];
                const uint32_t v = __builtin_amdgcn_alignbit(hi, lo, sh[j]);   // ({hi,lo} >> sh)[31:0]
                const int k0 = (int)__builtin_amdgcn_ubfe(v, 0u, b);
                const int k1 = (int)__builtin_amdgcn_ubfe(v, b, b);
                const int k2 = (int)__builtin_amdgcn_ubfe(v, 2u * b, b);
                const int k3 = (int)__builtin_amdgcn_ubfe(v, 3u * b, b);
                acc[j].x = __builtin_fmaf((float)(2 * k0 - (int)L), d, acc[j].x);
                acc[j].y = __builtin_fmaf((float)(2 * k1 - (int)L), d, acc[j].y);
                acc[j].z = __builtin_fmaf((float)(2 * k2 - (int)L), d, acc[j].z);
                acc[j].w = __builtin_fmaf((float)(2 * k3 - (int)L), d, acc[j].w);
            }
        }
    }

    // ---- a7: SGD step with the mean -----------------------------------------------------------
#pragma unroll
    for (int j = 0; j < kR; ++j) {
        const uint32_t el = 4u * (j * kThreads + tid);
        float4 r;
        r.x = __builtin_fmaf(a.neg_c, acc[j].x, x[j].x);
        r.y = __builtin_fmaf(a.neg_c, acc[j].y, x[j].y);
        r.z = __builtin_fmaf(a.neg_c, acc[j].z, x[j].z);
        r.w = __builtin_fmaf(a.neg_c, acc[j].w, x[j].w);
        if (full || el + 4u <= tile_count) {
            if (ALIGNED) {
                *reinterpret_cast<float4*>(p + el) = r;
            } else {
                p[el] = r.x; p[el + 1] = r.y; p[el + 2] = r.z; p[el + 3] = r.w;
            }
        } else {
            if (el + 0u < tile_count) p[el + 0] = r.x;
            if (el + 1u < tile_count) p[el + 1] = r.y;
            if (el + 2u < tile_count) p[el + 2] = r.z;
        }
    }
}

}  // namespace

hipError_t launch_aggregate(const AggregateArgs& a, hipStream_t stream) {
    if (a.n == 0) return hipSuccess;
    const uint64_t tiles = (a.n + kTile - 1) / kTile;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const bool aligned = (reinterpret_cast<uintptr_t>(a.params) & 15u) == 0;
    const dim3 grid((uint32_t)tiles), block(kThreads);
    if (aligned) {
        hipLaunchKernelGGL((aggregate_update_kernel<true>), grid, block, 0, stream, a);
    } else {
        hipLaunchKernelGGL((aggregate_update_kernel<false>), grid, block, 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace mqg
