// Internal launch interface between the C-ABI layer (api.hip) and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mqgrad.h"

namespace mqg {

struct QuantizeArgs {
    const float* grad;       // n floats
    uint64_t n;
    uint32_t bits;           // 1..8
    uint32_t bucket;         // multiple of 32, 32..16384
    int bucket_shift;        // log2(bucket) when bucket is a power of two, else -1
    int scale_mode;          // mqg_scale_mode
    uint32_t key0, key1;     // Philox key = seed
    uint32_t iteration, worker;
    uint64_t elem_base;      // multiple of 8
    const float* scales_in;  // nullable: when set, scales are read, not computed ([min, max] encoding: ONE
                             // (min, max) pair that holds for the whole tensor)
    uint32_t* packed;        // ceil(n*bits/32) words
    float* scales;           // ceil(n/bucket) floats
    uint32_t stream_codes = 0;   // 1: the code words are stored with the streaming hint instead of agent scope
};

struct AggregateArgs {
    const uint32_t* packed[MQG_MAX_WORKERS];
    const float* scales[MQG_MAX_WORKERS];
    uint32_t W;
    uint64_t n;
    uint32_t bits;
    uint32_t bucket;
    int bucket_shift;
    float neg_c;             // -(lr / W)
    float* params;
    uint32_t per_tensor;     // [min, max] encoding only: every worker has ONE (min, max) pair for the whole tensor
    uint32_t stream_codes;   // the code words are not in this GPU's caches: streaming loads at every width
};

// Server side of the full exchange: quantize the sum over W workers' de-quantized gradients
// (q.grad, q.scales_in unused); the stored bucket range is divided by W.
struct RequantArgs {
    QuantizeArgs q;
    const uint32_t* packed[MQG_MAX_WORKERS];
    const float* scales[MQG_MAX_WORKERS];
    uint32_t W;
};

// Several layer tensors of one model in one launch.
constexpr uint32_t kMaxBatchTensors = 32;
constexpr uint32_t kMaxBatchPointers = 256;   // per quantized tensor 2*W pointers, per raw tensor W

struct BatchAggregateArgs {
    struct Tensor {
        uint64_t n;
        float* params;
        uint32_t first_ptr;   // index into ptrs: [W packed][W scales], or [W raw gradients]
        uint32_t raw;         // 1: uncompressed layer
    };
    uint32_t count, W, bits, bucket;
    int bucket_shift;
    float neg_c;
    uint32_t per_tensor;      // [min, max] encoding only: ONE (min, max) pair per worker and tensor
    uint32_t tile_start[kMaxBatchTensors + 1];   // prefix sums of the tensors' tile counts
    Tensor t[kMaxBatchTensors];
    const void* ptrs[kMaxBatchPointers];
};

struct BatchQuantizeArgs {
    struct Tensor {
        const float* grad;
        uint64_t n;
        uint64_t elem_base;
        uint32_t* packed;
        float* scales;
        const float* scales_in;   // nullable: the layer's scales are read, not computed
    };
    QuantizeArgs common;      // bits, bucket, stream selection; per-tensor fields are taken from t[]
    uint32_t count;
    uint32_t tile_elems;
    uint32_t tile_start[kMaxBatchTensors + 1];
    Tensor t[kMaxBatchTensors];
};

uint32_t aggregate_batch_tile();
hipError_t launch_aggregate_tensors(const BatchAggregateArgs& a, uint32_t tiles, hipStream_t stream);
uint32_t quantize_batch_tile(const BatchQuantizeArgs& a);   // elements per workgroup of the kernel the batch will run (reads a.common only)
uint32_t quantize_wave_block_elems(uint32_t bucket, uint32_t bits);                             // quantize_wave.hip
hipError_t launch_quantize_tensors_wave(const BatchQuantizeArgs& a, uint32_t blocks, hipStream_t stream);
hipError_t launch_quantize_tensors(const BatchQuantizeArgs& a, uint32_t tiles, hipStream_t stream);

hipError_t launch_quantize(const QuantizeArgs& a, hipStream_t stream);
hipError_t launch_requantize(const RequantArgs& a, hipStream_t stream);
bool quantize_wave_supported(const QuantizeArgs& a);          // quantize_wave.hip
hipError_t launch_quantize_wave(const QuantizeArgs& a, hipStream_t stream);
bool quantize_cells_supported(const QuantizeArgs& a);         // quantize_wave.hip: other multiples of 32 up to 4064
hipError_t launch_quantize_cells(const QuantizeArgs& a, hipStream_t stream);
uint32_t quantize_cells_tile_elems(uint32_t bucket);
bool quantize_tensors_cells_supported(const BatchQuantizeArgs& a);
hipError_t launch_quantize_tensors_cells(const BatchQuantizeArgs& a, uint32_t tiles, hipStream_t stream);
bool quantize_minmax_wave_supported(const QuantizeArgs& a);   // quantize_wave.hip
hipError_t launch_quantize_minmax_wave(const QuantizeArgs& a, hipStream_t stream);
bool requantize_wave_supported(const RequantArgs& a);         // quantize_wave.hip
hipError_t launch_requantize_wave(const RequantArgs& a, hipStream_t stream);
hipError_t launch_aggregate(const AggregateArgs& a, hipStream_t stream);
hipError_t launch_aggregate_mean(const AggregateArgs& a, hipStream_t stream);   // a.params receives the mean gradient

// minmax.hip: deterministic [min, max] encoding; `scales` holds (min, max) pairs, 2 floats per bucket
hipError_t launch_quantize_minmax(const QuantizeArgs& a, hipStream_t stream);
hipError_t launch_aggregate_minmax(const AggregateArgs& a, hipStream_t stream);
hipError_t launch_requantize_minmax(const RequantArgs& a, hipStream_t stream);
hipError_t launch_requantize_minmax_tensor(const RequantArgs& a, hipStream_t stream);   // one range per worker and for the mean
hipError_t launch_tensor_range(const float* grad, uint64_t n, float* range_out, hipStream_t stream);
// the same for several layer tensors per launch
struct TensorRangeBatch {
    const float* grad[kMaxBatchTensors];
    uint64_t n[kMaxBatchTensors];
    float* range[kMaxBatchTensors];   // 2 floats each; nullptr: no such tensor (or an empty one)
};
hipError_t launch_tensor_range_batch(const TensorRangeBatch& b, uint32_t count, hipStream_t stream);
uint32_t quantize_minmax_wave_block_elems(uint32_t bucket);                                       // quantize_wave.hip
hipError_t launch_quantize_minmax_tensors_wave(const BatchQuantizeArgs& a, uint32_t blocks, hipStream_t stream);
uint32_t quantize_minmax_batch_tile(uint32_t bucket, int bucket_shift);   // elements per workgroup
hipError_t launch_quantize_minmax_tensors(const BatchQuantizeArgs& a, uint32_t tiles, hipStream_t stream);
uint32_t aggregate_minmax_batch_tile();
hipError_t launch_aggregate_minmax_tensors(const BatchAggregateArgs& a, uint32_t tiles, hipStream_t stream);
hipError_t launch_sum_squares(const float* grad, uint64_t n, double* out, hipStream_t stream);

// Sums of squares of several tensors in one launch, each added up in a fixed order.
constexpr uint32_t kMaxSumTensors = 64;
struct SumSquaresBatch {
    const float* grad[kMaxSumTensors];
    uint64_t n[kMaxSumTensors];
};
uint32_t sum_squares_batch_blocks();   // partial sums (doubles of scratch memory) per tensor
hipError_t launch_sum_squares_batch(const SumSquaresBatch& b, uint32_t count, double* partials, double* out, hipStream_t stream);
// the same with the partial sums in a device array the library holds (no allocation, no workspace argument)
hipError_t launch_sum_squares_batch_static(const SumSquaresBatch& b, uint32_t count, double* out, hipStream_t stream);

}  // namespace mqg
