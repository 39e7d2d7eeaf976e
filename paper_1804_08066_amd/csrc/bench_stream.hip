// Measurement aid, not part of libmqgrad: streaming kernels that move exactly the bytes of the two hot
// kernels, in the same launch shapes and with the same cache-policy hints, and do next to no
// arithmetic.  What they reach is what this machine's HBM gives to that read/write mix -- the practical
// ceiling that the benchmark sets the real kernels against (a device-to-device copy moves as many
// bytes out as in and is a poor stand-in for either kernel).
//
//   mqg_bench_stream_quantize   reads n floats, writes n * bits / 32 words        (mqg_quantize's mix)
//   mqg_bench_stream_update     reads W streams of n * bits / 32 words and n floats, writes n floats
//                               (mqg_aggregate_update's mix)
//   mqg_bench_stream_read / _write   a pure read and a pure write of n floats: the two rates from which the
//                               benchmark adds up the time a mix would take if reads and writes did not
//                               disturb each other
//
// Built into libmqgrad_bench.so, which only bench.py loads.  Sizes: n is rounded down to whole tiles by
// the caller (bench.py passes multiples of 8192); pointers are device pointers, 16-byte aligned.

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void store_v4u_agent(const void* base, uint32_t byte_off, v4u w) {
    asm volatile("global_store_dwordx4 %0, %1, %2 sc1" ::"v"(byte_off), "v"(w), "s"(base) : "memory");
}

// One wave per 256 * R floats (R float4 per lane, streaming loads), NW waves per workgroup; the wave
// writes its 8 * R * bits words with agent-scope 128-bit stores.  The stored words depend on every
// loaded value (a maximum over the wave), so no load can be dropped.
template <int R, int NW>
__global__ __launch_bounds__(64 * NW) void stream_quantize_kernel(const float* __restrict__ src, uint64_t n, uint32_t bits,
                                                                  uint32_t* __restrict__ dst) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint64_t chunk = (uint64_t)blockIdx.x * NW + wave;
    const uint64_t cb = chunk * (256u * R);
    if (cb + 256u * R > n) return;
    v4f x[R];
#pragma unroll
    for (int j = 0; j < R; ++j) x[j] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(src + cb + 4u * (j * 64u + lane)));
    float m = 0.0f;
#pragma unroll
    for (int j = 0; j < R; ++j) m = fmaxf(m, fmaxf(fmaxf(fabsf(x[j].x), fabsf(x[j].y)), fmaxf(fabsf(x[j].z), fabsf(x[j].w))));
    // every lane's values reach the lanes that store (fewer than 64 lanes store at low widths, and a load
    // whose value no store consumes would be dropped)
#pragma unroll
    for (int mask = 32; mask >= 1; mask >>= 1) m = fmaxf(m, __shfl_xor(m, mask, 64));
    const uint32_t mb = __builtin_bit_cast(uint32_t, m);
    const uint32_t* out = dst + chunk * (8u * R) * bits;
    for (uint32_t i = lane; i < 2u * R * bits; i += 64u) store_v4u_agent(out, 16u * i, v4u{mb, mb ^ i, mb + i, mb});
}

// One workgroup per 2048 parameters (2 float4 per lane, streaming loads and stores, as the server
// kernel moves them); each lane also reads, per worker and row, the dword that holds its quad's codes
// (a wave's request is one contiguous run of 32 * bits bytes; the loads of eight workers are issued
// together; streaming loads from 4 bits on, as in the server kernel).  All
// values are folded into what is stored.
constexpr int kMaxW = 64;
struct UpdateArgs {
    const uint32_t* codes[kMaxW];
    uint32_t W;
    uint32_t bits;
    uint64_t n;
    float* params;
};
// OCC: cap on the waves per SIMD.  With nothing to compute, eight waves per SIMD keep more requests in
// flight than HBM orders well: four are 5-6 % faster from 4 bits on (at 1 bit eight are).
template <bool ONCE, int OCC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, OCC))) void stream_update_kernel(const UpdateArgs a) {
    const uint32_t tid = threadIdx.x;
    const uint64_t tile = (uint64_t)blockIdx.x * 2048u;
    if (tile + 2048u > a.n) return;
    float* p = a.params + tile;
    v4f x[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) x[j] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p + 4u * (j * 256u + tid)));
    const uint64_t tile_word = (tile >> 5) * a.bits;
    const uint32_t w0 = (4u * a.bits * tid) >> 5, w1 = (4u * a.bits * (256u + tid)) >> 5;
    uint32_t acc = 0u;
    for (uint32_t wb = 0; wb < a.W; wb += 8u) {
        uint32_t c[8][2];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (wb + t < a.W) {
                const uint32_t* q = a.codes[wb + t] + tile_word;
                c[t][0] = ONCE ? __builtin_nontemporal_load(q + w0) : q[w0];
                c[t][1] = ONCE ? __builtin_nontemporal_load(q + w1) : q[w1];
            } else {
                c[t][0] = c[t][1] = 0u;
            }
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) acc ^= c[t][0] ^ c[t][1];
    }
    const float f = (acc == 0x9E3779B9u) ? 1.0f : 0.0f;   // practically never taken: the values pass through
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        v4f r = {x[j].x + f, x[j].y + f, x[j].z + f, x[j].w + f};
        __builtin_nontemporal_store(r, reinterpret_cast<v4f*>(p + 4u * (j * 256u + tid)));
    }
}

// Pure streams: 4096 floats per workgroup of 256 lanes, four float4 per lane, streaming hints.  What a
// kernel that only reads, or only writes, reaches on this machine.
__global__ __launch_bounds__(256) void stream_read_kernel(const float* __restrict__ src, uint64_t n, float* sink) {
    const uint64_t base = (uint64_t)blockIdx.x * 4096u;
    if (base + 4096u > n) return;
    v4f x[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) x[j] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(src + base + 4u * (j * 256u + threadIdx.x)));
    float m = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) m += (x[j].x + x[j].y) + (x[j].z + x[j].w);
    if (m == 1234.5678f) sink[threadIdx.x] = m;   // practically never taken: keeps the loads alive
}
__global__ __launch_bounds__(256) void stream_write_kernel(float* __restrict__ dst, uint64_t n) {
    const uint64_t base = (uint64_t)blockIdx.x * 4096u;
    if (base + 4096u > n) return;
    const v4f v = {1.0f, 2.0f, 3.0f, (float)blockIdx.x};
#pragma unroll
    for (int j = 0; j < 4; ++j) __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(dst + base + 4u * (j * 256u + threadIdx.x)));
}

}  // namespace

extern "C" {

// Read n floats (n a multiple of 4096); sink: device, 256 floats, practically never written.
int mqg_bench_stream_read(const float* src, uint64_t n, float* sink, void* stream) {
    if (n == 0) return 0;
    if (n % 4096u != 0u || n / 4096u > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(stream_read_kernel, dim3((uint32_t)(n / 4096u)), dim3(256), 0, (hipStream_t)stream, src, n, sink);
    return (int)hipGetLastError();
}
// Overwrite n floats (n a multiple of 4096).
int mqg_bench_stream_write(float* dst, uint64_t n, void* stream) {
    if (n == 0) return 0;
    if (n % 4096u != 0u || n / 4096u > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(stream_write_kernel, dim3((uint32_t)(n / 4096u)), dim3(256), 0, (hipStream_t)stream, dst, n);
    return (int)hipGetLastError();
}

// 0 on success, otherwise the hipError_t of the launch.  n must be a multiple of 8192, bits in 1..8.
// shape: 0 = 2048 floats per wave, 4 waves per workgroup (the quantizer's shape up to 7 bits);
//        1 = 1024 per wave, 4 waves (its shape at 8 bits);  2 = 2048 per wave, 2 waves.
int mqg_bench_stream_quantize(const float* src, uint64_t n, uint32_t bits, uint32_t shape, uint32_t* dst, void* stream) {
    if (n == 0) return 0;
    if (n % 8192u != 0u || bits < 1u || bits > 8u || shape > 2u || n / 2048u > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (shape == 0u) hipLaunchKernelGGL((stream_quantize_kernel<8, 4>), dim3((uint32_t)(n / 8192u)), dim3(256), 0, st, src, n, bits, dst);
    if (shape == 1u) hipLaunchKernelGGL((stream_quantize_kernel<4, 4>), dim3((uint32_t)(n / 4096u)), dim3(256), 0, st, src, n, bits, dst);
    if (shape == 2u) hipLaunchKernelGGL((stream_quantize_kernel<8, 2>), dim3((uint32_t)(n / 4096u)), dim3(128), 0, st, src, n, bits, dst);
    return (int)hipGetLastError();
}

// codes: HOST array of W device pointers, each to n * bits / 32 words.  n must be a multiple of 2048.
// shape: 0 = up to eight waves per SIMD, 1 = at most four.
int mqg_bench_stream_update(const uint32_t* const* codes, uint32_t W, uint64_t n, uint32_t bits, uint32_t shape, float* params,
                            void* stream) {
    if (n == 0) return 0;
    if (n % 2048u != 0u || bits < 1u || bits > 8u || shape > 1u || W < 1u || W > (uint32_t)kMaxW || n / 2048u > 0x7FFFFFFFull) {
        return (int)hipErrorInvalidValue;
    }
    UpdateArgs a;
    for (uint32_t w = 0; w < W; ++w) a.codes[w] = codes[w];
    for (uint32_t w = W; w < (uint32_t)kMaxW; ++w) a.codes[w] = nullptr;
    a.W = W;
    a.bits = bits;
    a.n = n;
    a.params = params;
    const dim3 grid((uint32_t)(n / 2048u)), block(256);
    hipStream_t st = (hipStream_t)stream;
    const bool once = bits >= 4u;   // the server kernel's rule: streaming loads of the code words from 4 bits on
    if (once && shape == 0u) hipLaunchKernelGGL((stream_update_kernel<true, 8>), grid, block, 0, st, a);
    if (once && shape == 1u) hipLaunchKernelGGL((stream_update_kernel<true, 4>), grid, block, 0, st, a);
    if (!once && shape == 0u) hipLaunchKernelGGL((stream_update_kernel<false, 8>), grid, block, 0, st, a);
    if (!once && shape == 1u) hipLaunchKernelGGL((stream_update_kernel<false, 4>), grid, block, 0, st, a);
    return (int)hipGetLastError();
}

}  // extern "C"
