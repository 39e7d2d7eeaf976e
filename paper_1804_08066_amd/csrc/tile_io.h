// Streaming tile loads and stores of fp32 parameters (step a7 of the hot path), shared by the server
// kernels: a workgroup of 256 lanes owns R rows of 1024 consecutive values, one float4 per lane and row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mqg {
namespace tile_io {

constexpr int kThreads = 256;

typedef float v4f __attribute__((ext_vector_type(4)));
// Global memory takes multi-dword accesses at any dword address: a tensor that starts off a 16-byte
// boundary is still read and written 128 bits at a time (a wave's row then touches nine 128-byte lines
// instead of eight).
typedef v4f v4f_a4 __attribute__((aligned(4)));

__device__ __forceinline__ float4 load_f4_stream(const float* p) {
    const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f_a4*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void store_f4_stream(float* p, const float4& r) {
    v4f t = {r.x, r.y, r.z, r.w};
    __builtin_nontemporal_store(t, reinterpret_cast<v4f_a4*>(p));
}

template <int R>
__device__ __forceinline__ void load_params(const float* __restrict__ p, uint32_t tile_count, bool full,
                                            float4 (&x)[R]) {
    const uint32_t tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t el = 4u * (j * kThreads + tid);
        if (full || el + 4u <= tile_count) {
            x[j] = load_f4_stream(p + el);
        } else {
            x[j].x = (el + 0u < tile_count) ? p[el + 0] : 0.0f;
            x[j].y = (el + 1u < tile_count) ? p[el + 1] : 0.0f;
            x[j].z = (el + 2u < tile_count) ? p[el + 2] : 0.0f;
            x[j].w = 0.0f;   // el + 3 >= tile_count here
        }
    }
}

// a7: p <- fma(-(lr/W), acc, p)
template <int R>
__device__ __forceinline__ void update_params(float* __restrict__ p, uint32_t tile_count, bool full, float neg_c,
                                              const float4 (&x)[R], const float4 (&acc)[R]) {
    const uint32_t tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t el = 4u * (j * kThreads + tid);
        float4 r;
        r.x = __builtin_fmaf(neg_c, acc[j].x, x[j].x);
        r.y = __builtin_fmaf(neg_c, acc[j].y, x[j].y);
        r.z = __builtin_fmaf(neg_c, acc[j].z, x[j].z);
        r.w = __builtin_fmaf(neg_c, acc[j].w, x[j].w);
        if (full || el + 4u <= tile_count) {
            store_f4_stream(p + el, r);
        } else {
            if (el + 0u < tile_count) p[el + 0] = r.x;
            if (el + 1u < tile_count) p[el + 1] = r.y;
            if (el + 2u < tile_count) p[el + 2] = r.z;
        }
    }
}

// An uncompressed layer: acc <- sum over the W workers' fp32 gradients of the tile, in worker order.
template <int R>
__device__ __forceinline__ void accumulate_raw(const float* const* raw, uint32_t W, uint64_t tile_base, uint32_t tile_count,
                                               bool full, float4 (&acc)[R]) {
    const uint32_t tid = threadIdx.x;
    for (uint32_t w = 0; w < W; ++w) {
        const float* __restrict__ g = raw[w] + tile_base;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint32_t el = 4u * (j * kThreads + tid);
            if (full || el + 4u <= tile_count) {
                const float4 t = load_f4_stream(g + el);
                acc[j].x = acc[j].x + t.x;
                acc[j].y = acc[j].y + t.y;
                acc[j].z = acc[j].z + t.z;
                acc[j].w = acc[j].w + t.w;
            } else {
                if (el + 0u < tile_count) acc[j].x = acc[j].x + g[el + 0];
                if (el + 1u < tile_count) acc[j].y = acc[j].y + g[el + 1];
                if (el + 2u < tile_count) acc[j].z = acc[j].z + g[el + 2];
            }
        }
    }
}

}  // namespace tile_io
}  // namespace mqg
