// Worker side of MQGrad's hot path on gfx950: Quantize(g, K) of Algorithm 1 (WorkerIterate),
// the range-linear K-bit encode of the Section 3.2 footnote, done in ONE pass over the gradient:
//
//   a1  per-bucket range  s = max |g|            (DPP max over 8-lane cells, LDS max per bucket)
//   a2  position on the 2^K-level grid           u = clamp(fma(g, (L/2)/s, L/2), 0, L)
//   a3  stochastic rounding with Philox4x32-10   c = floor(u) + [(h + 1/2)/65536 < frac(u)]
//   a4  dense little-endian bit packing          LDS-staged, whole words stored coalesced
//
// Work decomposition.  A workgroup of 256 lanes owns one tile = a whole number of buckets, at most
// CAP = 1024*R elements, and keeps it in registers (R float4 per lane) between the range
// reduction and the rounding, so each gradient byte is read from HBM exactly once.  Row j of a
// tile is the 1024 consecutive elements that the 256 lanes load with one float4 each; 8
// consecutive lanes hold a 32-element "cell", which never straddles a bucket (buckets are
// multiples of 32) and packs into exactly `bits` words.
//
// Random numbers.  One Philox call yields 8 16-bit uniforms for 8 consecutive elements, i.e. for
// the quads of an even/odd lane pair.  So that no lane computes a call whose output is thrown
// away, the even lane computes the pair's call for row j and the odd lane the call for row j+1;
// they swap halves with one DPP quad permute per word.

#include "kernels.h"

namespace mqg {
namespace {

constexpr int kThreads = 256;
constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;

constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]: lane ^ 1
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]: lane ^ 2
constexpr int kDppRowHalfMirror = 0x141; // lane i <-> 7 - i inside each group of 8

typedef float v4f __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __builtin_bit_cast(float, dpp_u32<CTRL>(__builtin_bit_cast(uint32_t, v)));
}

// Philox4x32-10 (Salmon et al., SC'11).  Ten rounds of two 32x32->64 multiplies; the key is
// bumped by the Weyl constants between rounds.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&o)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
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

template <int R>
struct Tile {
    static constexpr uint32_t kCap = 1024u * R;           // elements
    static constexpr uint32_t kMaxWords = kCap * 8u / 32u; // at 8 bits
};

template <int R, bool ALIGNED, bool FULL>
__device__ __forceinline__ void quantize_tile(const QuantizeArgs& a, const uint64_t tile_base,
                                              const uint32_t tile_count, uint32_t* s_words,
                                              uint32_t* s_bmax, float* s_ainv, float* s_cellsq) {
    const uint32_t tid = threadIdx.x;
    const float* __restrict__ g = a.grad + tile_base;

    // ---- load the tile (one HBM pass) -------------------------------------------------------
    float4 x[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t el = 4u * (j * kThreads + tid);
        if (FULL || el + 4u <= tile_count) {
            if (ALIGNED) {
                const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(g + el));   // read once: streaming
                x[j] = make_float4(t.x, t.y, t.z, t.w);
            } else {
                x[j] = make_float4(g[el], g[el + 1], g[el + 2], g[el + 3]);
            }
        } else {
            x[j].x = (el + 0u < tile_count) ? g[el + 0] : 0.0f;
            x[j].y = (el + 1u < tile_count) ? g[el + 1] : 0.0f;
            x[j].z = (el + 2u < tile_count) ? g[el + 2] : 0.0f;
            x[j].w = 0.0f;  // el + 3 >= tile_count here
        }
    }

    // ---- clear the LDS staging while the loads are in flight -------------------------------
    const uint32_t nwords = (tile_count * a.bits + 31u) >> 5;
    for (uint32_t i = tid; i < nwords; i += kThreads) s_words[i] = 0u;
    if (tid < 128u) s_bmax[tid] = 0u;
    __syncthreads();

    const uint32_t nbt = (R > 4) ? 1u : (tile_count + a.bucket - 1u) / a.bucket;  // buckets in tile
    const uint64_t kb0 = tile_base / a.bucket;

    // ---- a1: bucket range -------------------------------------------------------------------
    uint32_t bl[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        const uint32_t el = 4u * (j * kThreads + tid);
        bl[j] = (R > 4) ? 0u : (a.bucket_shift >= 0 ? (el >> a.bucket_shift) : (el / a.bucket));
    }
    if (a.scales_in == nullptr) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint32_t el = 4u * (j * kThreads + tid);
            float m = fmaxf(fmaxf(fabsf(x[j].x), fabsf(x[j].y)), fmaxf(fabsf(x[j].z), fabsf(x[j].w)));
            m = fmaxf(m, dpp_f32<kDppQuadSwap1>(m));
            m = fmaxf(m, dpp_f32<kDppQuadSwap2>(m));
            m = fmaxf(m, dpp_f32<kDppRowHalfMirror>(m));
            if ((tid & 7u) == 0u && (FULL || el < tile_count)) {
                atomicMax(&s_bmax[bl[j]], __builtin_bit_cast(uint32_t, m));  // m >= 0: bit order = value order
            }
        }
        if (a.scale_mode == MQG_SCALE_L2) {
            // sum of squares of each 32-element cell, in a fixed order (reproducible)
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const uint32_t ql = j * kThreads + tid;
                float q = (x[j].x * x[j].x + x[j].y * x[j].y) + (x[j].z * x[j].z + x[j].w * x[j].w);
                q += dpp_f32<kDppQuadSwap1>(q);
                q += dpp_f32<kDppQuadSwap2>(q);
                q += dpp_f32<kDppRowHalfMirror>(q);
                if ((tid & 7u) == 0u) s_cellsq[ql >> 3] = q;   // zero for cells past the end
            }
        }
    }
    __syncthreads();
    if (a.scales_in == nullptr && a.scale_mode == MQG_SCALE_L2) {
        // one wave per bucket: lanes add the bucket's cell sums (stride 64) in fp64, then a
        // butterfly over the wave; the norm is raised to max|g| if rounding left it below
        const uint32_t nbt_l2 = (R > 4) ? 1u : (tile_count + a.bucket - 1u) / a.bucket;
        const uint32_t cpb = a.bucket >> 5;
        const uint32_t lane = tid & 63u;
        for (uint32_t k = tid >> 6; k < nbt_l2; k += kThreads / 64) {
            double acc = 0.0;
            for (uint32_t c = lane; c < cpb; c += 64u) acc += (double)s_cellsq[k * cpb + c];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
            if (lane == 0u) {
                const float norm = (float)__builtin_sqrt(acc);
                const float mx = __builtin_bit_cast(float, s_bmax[k]);
                s_bmax[k] = __builtin_bit_cast(uint32_t, norm < mx ? mx : norm);
            }
        }
        __syncthreads();
    }

    const float Lf = (float)((1u << a.bits) - 1u);
    const float halfL = 0.5f * Lf;
    if (tid < nbt) {
        float s;
        if (a.scales_in != nullptr) {
            s = a.scales_in[kb0 + tid];
        } else {
            s = __builtin_bit_cast(float, s_bmax[tid]);
            if (!(s >= 0x1p-96f)) s = 0.0f;
        }
        a.scales[kb0 + tid] = s;
        s_ainv[tid] = (s > 0.0f) ? halfL / s : 0.0f;   // IEEE-correct fp32 division, once per bucket
    }
    __syncthreads();

    // ---- a2..a4: grid position, stochastic rounding, packing --------------------------------
    const uint32_t odd = tid & 1u;
    const uint64_t group0 = (a.elem_base + tile_base) >> 3;  // both multiples of 8
    const uint32_t b = a.bits;
    const uint32_t cell_bit = 4u * b * (tid & 7u);           // this lane's bit offset in its cell
    const uint32_t sh = cell_bit & 31u;
    const uint32_t word_in_cell = cell_bit >> 5;
    const bool straddle = sh + 4u * b > 32u;

#pragma unroll
    for (int jp = 0; jp < R; jp += 2) {
        // the even lane draws for row jp, the odd lane for row jp + 1
        const uint32_t my_row = jp + odd;
        const uint64_t grp = group0 + (uint64_t)((my_row * kThreads + tid) >> 1);
        uint32_t o[4];
        philox4x32_10((uint32_t)grp, (uint32_t)(grp >> 32), a.iteration, a.worker, a.key0, a.key1, o);
        // an even lane keeps words 0,1 and gives away 2,3; an odd lane keeps 2,3 and gives away 0,1
        const uint32_t keep0 = odd ? o[2] : o[0];
        const uint32_t keep1 = odd ? o[3] : o[1];
        const uint32_t got0 = dpp_u32<kDppQuadSwap1>(odd ? o[0] : o[2]);
        const uint32_t got1 = dpp_u32<kDppQuadSwap1>(odd ? o[1] : o[3]);
        // row jp uses the even lane's call, row jp+1 the odd lane's
        const uint32_t rw[2][2] = {{odd ? got0 : keep0, odd ? got1 : keep1},
                                   {odd ? keep0 : got0, odd ? keep1 : got1}};
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int j = jp + t;
            const uint32_t ql = j * kThreads + tid;
            const uint32_t el = 4u * ql;
            const float ainv = s_ainv[bl[j]];
            uint32_t k0 = round_code(x[j].x, ainv, halfL, Lf, rw[t][0] & 0xFFFFu);
            uint32_t k1 = round_code(x[j].y, ainv, halfL, Lf, rw[t][0] >> 16);
            uint32_t k2 = round_code(x[j].z, ainv, halfL, Lf, rw[t][1] & 0xFFFFu);
            uint32_t k3 = round_code(x[j].w, ainv, halfL, Lf, rw[t][1] >> 16);
            if (!FULL) {   // elements past the end contribute zero bits
                if (el + 0u >= tile_count) k0 = 0u;
                if (el + 1u >= tile_count) k1 = 0u;
                if (el + 2u >= tile_count) k2 = 0u;
                if (el + 3u >= tile_count) k3 = 0u;
            }
            const uint32_t v = k0 | (k1 << b) | (k2 << (2u * b)) | (k3 << (3u * b));
            if (FULL || el < tile_count) {
                const uint32_t w0 = (ql >> 3) * b + word_in_cell;
                atomicOr(&s_words[w0], v << sh);
                if (straddle) atomicOr(&s_words[w0 + 1u], v >> (32u - sh));
            }
        }
    }
    __syncthreads();

    // ---- store whole words, coalesced -------------------------------------------------------
    uint32_t* __restrict__ out = a.packed + (tile_base >> 5) * b;
    for (uint32_t i = tid; i < nwords; i += kThreads) __builtin_nontemporal_store(s_words[i], out + i);
}

template <int R, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void quantize_pack_kernel(const QuantizeArgs a, const uint32_t tile_elems) {
    __shared__ uint32_t s_words[Tile<R>::kMaxWords + 4];
    __shared__ uint32_t s_bmax[128];
    __shared__ float s_ainv[128];
    __shared__ float s_cellsq[Tile<R>::kCap / 32u];
    const uint64_t tile_base = (uint64_t)blockIdx.x * tile_elems;
    const uint64_t left = a.n - tile_base;
    const uint32_t tile_count = left < tile_elems ? (uint32_t)left : tile_elems;
    if (tile_count == Tile<R>::kCap) {
        quantize_tile<R, ALIGNED, true>(a, tile_base, tile_count, s_words, s_bmax, s_ainv, s_cellsq);
    } else {
        quantize_tile<R, ALIGNED, false>(a, tile_base, tile_count, s_words, s_bmax, s_ainv, s_cellsq);
    }
}

template <int R>
hipError_t launch_r(const QuantizeArgs& a, hipStream_t stream) {
    const uint32_t cap = Tile<R>::kCap;
    const uint32_t tile_elems = (cap / a.bucket) * a.bucket;   // whole buckets, >= 1 by choice of R
    const uint64_t tiles = (a.n + tile_elems - 1) / tile_elems;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const bool aligned = (reinterpret_cast<uintptr_t>(a.grad) & 15u) == 0;
    const dim3 grid((uint32_t)tiles), block(kThreads);
    if (aligned) {
        hipLaunchKernelGGL((quantize_pack_kernel<R, true>), grid, block, 0, stream, a, tile_elems);
    } else {
        hipLaunchKernelGGL((quantize_pack_kernel<R, false>), grid, block, 0, stream, a, tile_elems);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_quantize(const QuantizeArgs& a, hipStream_t stream) {
    if (a.n == 0) return hipSuccess;
    if (quantize_wave_supported(a)) return launch_quantize_wave(a, stream);
    if (a.bucket <= 4096u) return launch_r<4>(a, stream);
    if (a.bucket <= 8192u) return launch_r<8>(a, stream);
    return launch_r<16>(a, stream);
}

}  // namespace mqg
