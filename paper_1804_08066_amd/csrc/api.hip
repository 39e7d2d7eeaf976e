// C-ABI layer of libmqgrad: argument validation and launch set-up.  No arithmetic of the method
// happens here; the kernels are in quantize_pack.hip, quantize_wave.hip, aggregate_update.hip and minmax.hip.

#include "kernels.h"

namespace {

bool valid_common(uint32_t bits, uint32_t bucket) {
    return bits >= 1u && bits <= 8u && bucket >= MQG_MIN_BUCKET && bucket <= MQG_MAX_BUCKET &&
           (bucket % 32u) == 0u;
}

int log2_if_pow2(uint32_t v) {
    if (v == 0u || (v & (v - 1u)) != 0u) return -1;
    int s = 0;
    while ((1u << s) != v) ++s;
    return s;
}

bool misaligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) != 0; }
bool misaligned8(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 7u) != 0; }

mqg_status quantize_impl(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket, int mode,
                         uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                         const float* scales_in, bool use_scales_in, uint32_t* packed_out,
                         float* scales_out, void* stream, bool stream_codes = false) {
    if (!valid_common(bits, bucket)) return MQG_EINVAL;
    if ((elem_base & 7u) != 0u) return MQG_EINVAL;
    if (mode != MQG_SCALE_MAXABS && mode != MQG_SCALE_L2) return MQG_EINVAL;
    if (n == 0) return MQG_OK;
    if (grad == nullptr || packed_out == nullptr || scales_out == nullptr) return MQG_EINVAL;
    if (use_scales_in && scales_in == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4) || elem_base > UINT64_MAX - n) return MQG_EINVAL;
    if (misaligned4(grad) || misaligned4(packed_out) || misaligned4(scales_out) ||
        (use_scales_in && misaligned4(scales_in)))
        return MQG_EALIGN;

    mqg::QuantizeArgs a;
    a.grad = grad;
    a.n = n;
    a.bits = bits;
    a.bucket = bucket;
    a.bucket_shift = log2_if_pow2(bucket);
    a.scale_mode = mode;
    a.key0 = (uint32_t)seed;
    a.key1 = (uint32_t)(seed >> 32);
    a.iteration = iteration;
    a.worker = worker;
    a.elem_base = elem_base;
    a.scales_in = use_scales_in ? scales_in : nullptr;
    a.packed = packed_out;
    a.scales = scales_out;
    a.stream_codes = stream_codes ? 1u : 0u;
    const hipError_t err = mqg::launch_quantize(a, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

// shared argument checks of the two batched forms; fills b
mqg_status sumsq_batch_args(const mqg_sumsq_item* items, uint32_t count, const double* sumsq_out, mqg::SumSquaresBatch& b) {
    if (items == nullptr || sumsq_out == nullptr || count > MQG_MAX_SUMSQ_TENSORS) return MQG_EINVAL;
    for (uint32_t k = 0; k < count; ++k) {
        if (items[k].n > 0 && items[k].grad == nullptr) return MQG_EINVAL;
        if (items[k].n > (UINT64_MAX >> 4)) return MQG_EINVAL;
        if (items[k].n > 0 && misaligned4(items[k].grad)) return MQG_EALIGN;
        b.grad[k] = items[k].grad;
        b.n[k] = items[k].n;
    }
    for (uint32_t k = count; k < mqg::kMaxSumTensors; ++k) {
        b.grad[k] = nullptr;
        b.n[k] = 0;
    }
    if (misaligned8(sumsq_out)) return MQG_EALIGN;
    return MQG_OK;
}

// The W workers' stream and scale pointers of a server call into a launch table (slots past W cleared).
// `pairs`: the scale arrays hold (min, max) pairs and must be 8-byte aligned.
mqg_status worker_tables(const uint32_t* const* packed, const float* const* scales, uint32_t W, bool pairs,
                         const uint32_t* (&packed_tab)[MQG_MAX_WORKERS], const float* (&scales_tab)[MQG_MAX_WORKERS]) {
    for (uint32_t w = 0; w < MQG_MAX_WORKERS; ++w) {
        packed_tab[w] = nullptr;
        scales_tab[w] = nullptr;
    }
    for (uint32_t w = 0; w < W; ++w) {
        if (packed[w] == nullptr || scales[w] == nullptr) return MQG_EINVAL;
        if (misaligned4(packed[w]) || (pairs ? misaligned8(scales[w]) : misaligned4(scales[w]))) return MQG_EALIGN;
        packed_tab[w] = packed[w];
        scales_tab[w] = scales[w];
    }
    return MQG_OK;
}

// Fills the launch table of a batched server step; `minmax`: the scale arrays hold (min, max) pairs and
// must be 8-byte aligned.  MQG_OK with *tiles_out == 0 when there is nothing to do.
mqg_status update_batch_args(const mqg_update_item* items, uint32_t count, uint32_t W, uint32_t bits,
                                    uint32_t bucket, float lr, bool minmax, uint32_t tile,
                                    mqg::BatchAggregateArgs& a, uint32_t* tiles_out) {
    *tiles_out = 0;
    if (W < 1u || W > MQG_MAX_WORKERS) return MQG_EINVAL;
    if (count > MQG_MAX_TENSORS) return MQG_EINVAL;
    if (count == 0) return MQG_OK;
    if (items == nullptr) return MQG_EINVAL;
    a.count = count;
    a.W = W;
    a.bits = bits;
    a.bucket = bucket;
    a.bucket_shift = log2_if_pow2(bucket);
    a.neg_c = -(lr / (float)W);
    a.per_tensor = 0u;
    for (uint32_t i = 0; i < mqg::kMaxBatchPointers; ++i) a.ptrs[i] = nullptr;
    uint64_t tiles = 0;
    uint32_t used = 0;
    for (uint32_t i = 0; i < mqg::kMaxBatchTensors; ++i) {
        a.tile_start[i] = (uint32_t)tiles;
        a.t[i] = mqg::BatchAggregateArgs::Tensor{0, nullptr, 0, 0};
        if (i >= count) continue;
        const mqg_update_item& it = items[i];
        if (it.n == 0) continue;
        if (it.params == nullptr || it.n > (UINT64_MAX >> 4)) return MQG_EINVAL;
        if (misaligned4(it.params)) return MQG_EALIGN;
        const bool raw = it.packed == nullptr;
        const uint32_t need = raw ? W : 2u * W;
        if (used + need > mqg::kMaxBatchPointers) return MQG_EINVAL;
        if (raw) {
            if (it.raw == nullptr) return MQG_EINVAL;
            for (uint32_t w = 0; w < W; ++w) {
                if (it.raw[w] == nullptr) return MQG_EINVAL;
                if (misaligned4(it.raw[w])) return MQG_EALIGN;
                a.ptrs[used + w] = it.raw[w];
            }
        } else {
            if (it.scales == nullptr) return MQG_EINVAL;
            for (uint32_t w = 0; w < W; ++w) {
                if (it.packed[w] == nullptr || it.scales[w] == nullptr) return MQG_EINVAL;
                if (misaligned4(it.packed[w]) || (minmax ? misaligned8(it.scales[w]) : misaligned4(it.scales[w]))) return MQG_EALIGN;
                a.ptrs[used + w] = it.packed[w];
                a.ptrs[used + W + w] = it.scales[w];
            }
        }
        a.t[i] = mqg::BatchAggregateArgs::Tensor{it.n, it.params, used, raw ? 1u : 0u};
        used += need;
        tiles += (it.n + tile - 1) / tile;
        if (tiles > 0x7FFFFFFFull) return MQG_EINVAL;
    }
    a.tile_start[mqg::kMaxBatchTensors] = (uint32_t)tiles;
    *tiles_out = (uint32_t)tiles;
    return MQG_OK;
}

}  // namespace

extern "C" {

const char* mqg_status_string(mqg_status st) {
    switch (st) {
        case MQG_OK: return "MQG_OK";
        case MQG_EINVAL: return "MQG_EINVAL: argument out of range or NULL";
        case MQG_EALIGN: return "MQG_EALIGN: pointer not aligned as required";
        case MQG_ELAUNCH: return "MQG_ELAUNCH: HIP launch failed";
    }
    return "MQG: unknown status";
}

size_t mqg_num_buckets(uint64_t n, uint32_t bucket) {
    if (bucket == 0u) return 0;
    return (size_t)(n / bucket + (n % bucket != 0u ? 1u : 0u));
}

size_t mqg_packed_words(uint64_t n, uint32_t bits) {
    if (bits == 0u) return 0;
    // n * bits without overflow for any n: split n into whole 32-element cells and the rest
    const uint64_t cells = n >> 5, rest = n & 31u;
    return (size_t)(cells * bits + ((rest * bits + 31u) >> 5));
}

mqg_status mqg_quantize(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket,
                        uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                        uint32_t* packed_out, float* scales_out, void* stream) {
    return quantize_impl(grad, n, bits, bucket, MQG_SCALE_MAXABS, seed, iteration, worker, elem_base,
                         nullptr, false, packed_out, scales_out, stream);
}

mqg_status mqg_quantize_to(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket,
                           uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                           uint32_t* packed_out, float* scales_out, mqg_codes_destination dest, void* stream) {
    if (dest != MQG_CODES_KEEP_CACHED && dest != MQG_CODES_TO_MEMORY) return MQG_EINVAL;
    return quantize_impl(grad, n, bits, bucket, MQG_SCALE_MAXABS, seed, iteration, worker, elem_base,
                         nullptr, false, packed_out, scales_out, stream, dest == MQG_CODES_TO_MEMORY);
}

mqg_status mqg_quantize_mode(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket,
                             mqg_scale_mode mode,
                             uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                             uint32_t* packed_out, float* scales_out, void* stream) {
    return quantize_impl(grad, n, bits, bucket, (int)mode, seed, iteration, worker, elem_base,
                         nullptr, false, packed_out, scales_out, stream);
}

mqg_status mqg_quantize_with_scales(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket,
                                    uint64_t seed, uint32_t iteration, uint32_t worker,
                                    uint64_t elem_base, const float* scales_in,
                                    uint32_t* packed_out, float* scales_out, void* stream) {
    return quantize_impl(grad, n, bits, bucket, MQG_SCALE_MAXABS, seed, iteration, worker, elem_base,
                         scales_in, true, packed_out, scales_out, stream);
}

mqg_status mqg_aggregate_update(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                                uint64_t n, uint32_t bits, uint32_t bucket,
                                float lr, float* params, void* stream) {
    return mqg_aggregate_update_from(packed, scales, W, n, bits, bucket, lr, params, MQG_CODES_MAY_BE_CACHED, stream);
}

mqg_status mqg_aggregate_update_from(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                                     uint64_t n, uint32_t bits, uint32_t bucket,
                                     float lr, float* params, mqg_codes_origin origin, void* stream) {
    if (origin != MQG_CODES_MAY_BE_CACHED && origin != MQG_CODES_FROM_MEMORY) return MQG_EINVAL;
    if (!valid_common(bits, bucket)) return MQG_EINVAL;
    if (W < 1u || W > MQG_MAX_WORKERS) return MQG_EINVAL;
    if (n == 0) return MQG_OK;
    if (packed == nullptr || scales == nullptr || params == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4)) return MQG_EINVAL;
    if (misaligned4(params)) return MQG_EALIGN;
    mqg::AggregateArgs a;
    a.stream_codes = origin == MQG_CODES_FROM_MEMORY ? 1u : 0u;
    const mqg_status tables = worker_tables(packed, scales, W, false, a.packed, a.scales);
    if (tables != MQG_OK) return tables;
    a.W = W;
    a.n = n;
    a.bits = bits;
    a.bucket = bucket;
    a.bucket_shift = log2_if_pow2(bucket);
    a.neg_c = -(lr / (float)W);
    a.params = params;
    a.per_tensor = 0u;
    const hipError_t err = mqg::launch_aggregate(a, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_aggregate_mean(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                              uint64_t n, uint32_t bits, uint32_t bucket,
                              float* mean_out, void* stream) {
    if (!valid_common(bits, bucket)) return MQG_EINVAL;
    if (W < 1u || W > MQG_MAX_WORKERS) return MQG_EINVAL;
    if (n == 0) return MQG_OK;
    if (packed == nullptr || scales == nullptr || mean_out == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4)) return MQG_EINVAL;
    if (misaligned4(mean_out)) return MQG_EALIGN;
    mqg::AggregateArgs a;
    a.stream_codes = 0u;
    const mqg_status tables = worker_tables(packed, scales, W, false, a.packed, a.scales);
    if (tables != MQG_OK) return tables;
    a.W = W;
    a.n = n;
    a.bits = bits;
    a.bucket = bucket;
    a.bucket_shift = log2_if_pow2(bucket);
    a.neg_c = 0.0f;
    a.params = mean_out;
    a.per_tensor = 0u;
    const hipError_t err = mqg::launch_aggregate_mean(a, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_aggregate_requantize(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                                    uint64_t n, uint32_t bits, uint32_t bucket,
                                    uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                                    uint32_t* packed_out, float* scales_out, void* stream) {
    return mqg_aggregate_requantize_mode(packed, scales, W, n, bits, bucket, MQG_SCALE_MAXABS, seed, iteration, worker,
                                         elem_base, packed_out, scales_out, stream);
}

mqg_status mqg_aggregate_requantize_mode(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                                         uint64_t n, uint32_t bits, uint32_t bucket, mqg_scale_mode mode,
                                         uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                                         uint32_t* packed_out, float* scales_out, void* stream) {
    if (!valid_common(bits, bucket)) return MQG_EINVAL;
    if (mode != MQG_SCALE_MAXABS && mode != MQG_SCALE_L2) return MQG_EINVAL;
    if (W < 1u || W > MQG_MAX_WORKERS) return MQG_EINVAL;
    if ((elem_base & 7u) != 0u) return MQG_EINVAL;
    if (n == 0) return MQG_OK;
    if (packed == nullptr || scales == nullptr || packed_out == nullptr || scales_out == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4) || elem_base > UINT64_MAX - n) return MQG_EINVAL;
    if (misaligned4(packed_out) || misaligned4(scales_out)) return MQG_EALIGN;
    mqg::RequantArgs ra;
    const mqg_status tables = worker_tables(packed, scales, W, false, ra.packed, ra.scales);
    if (tables != MQG_OK) return tables;
    ra.W = W;
    ra.q.grad = nullptr;
    ra.q.n = n;
    ra.q.bits = bits;
    ra.q.bucket = bucket;
    ra.q.bucket_shift = log2_if_pow2(bucket);
    ra.q.scale_mode = mode;
    ra.q.key0 = (uint32_t)seed;
    ra.q.key1 = (uint32_t)(seed >> 32);
    ra.q.iteration = iteration;
    ra.q.worker = worker;
    ra.q.elem_base = elem_base;
    ra.q.scales_in = nullptr;
    ra.q.packed = packed_out;
    ra.q.scales = scales_out;
    const hipError_t err = mqg::launch_requantize(ra, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_dequantize_update(const uint32_t* packed, const float* scales, uint64_t n, uint32_t bits,
                                 uint32_t bucket, float lr, float* params, void* stream) {
    const uint32_t* pk[1] = {packed};
    const float* sc[1] = {scales};
    return mqg_aggregate_update(pk, sc, 1u, n, bits, bucket, lr, params, stream);
}

mqg_status mqg_quantize_tensors(const mqg_quantize_item* items, uint32_t count, uint32_t bits, uint32_t bucket,
                                uint64_t seed, uint32_t iteration, uint32_t worker, void* stream) {
    return mqg_quantize_tensors_mode(items, count, bits, bucket, MQG_SCALE_MAXABS, seed, iteration, worker, stream);
}

mqg_status mqg_quantize_tensors_mode(const mqg_quantize_item* items, uint32_t count, uint32_t bits, uint32_t bucket,
                                     mqg_scale_mode mode, uint64_t seed, uint32_t iteration, uint32_t worker,
                                     void* stream) {
    if (!valid_common(bits, bucket)) return MQG_EINVAL;
    if (mode != MQG_SCALE_MAXABS && mode != MQG_SCALE_L2) return MQG_EINVAL;
    if (count > MQG_MAX_TENSORS) return MQG_EINVAL;
    if (count == 0) return MQG_OK;
    if (items == nullptr) return MQG_EINVAL;
    mqg::BatchQuantizeArgs a;
    a.common.grad = nullptr;
    a.common.n = 0;
    a.common.bits = bits;
    a.common.bucket = bucket;
    a.common.bucket_shift = log2_if_pow2(bucket);
    a.common.scale_mode = mode;
    a.common.key0 = (uint32_t)seed;
    a.common.key1 = (uint32_t)(seed >> 32);
    a.common.iteration = iteration;
    a.common.worker = worker;
    a.common.elem_base = 0;
    a.common.scales_in = nullptr;
    a.common.packed = nullptr;
    a.common.scales = nullptr;
    a.count = count;
    a.tile_elems = mqg::quantize_batch_tile(a);
    uint64_t tiles = 0;
    for (uint32_t i = 0; i < mqg::kMaxBatchTensors; ++i) {
        a.tile_start[i] = (uint32_t)tiles;
        mqg::BatchQuantizeArgs::Tensor& t = a.t[i];
        t = mqg::BatchQuantizeArgs::Tensor{nullptr, 0, 0, nullptr, nullptr, nullptr};
        if (i >= count) continue;
        const mqg_quantize_item& it = items[i];
        if ((it.elem_base & 7u) != 0u) return MQG_EINVAL;
        if (it.n == 0) continue;
        if (it.grad == nullptr || it.packed_out == nullptr || it.scales_out == nullptr) return MQG_EINVAL;
        if (it.n > (UINT64_MAX >> 4) || it.elem_base > UINT64_MAX - it.n) return MQG_EINVAL;
        if (misaligned4(it.grad) || misaligned4(it.packed_out) || misaligned4(it.scales_out) || misaligned4(it.scales_in)) {
            return MQG_EALIGN;
        }
        t = mqg::BatchQuantizeArgs::Tensor{it.grad, it.n, it.elem_base, it.packed_out, it.scales_out, it.scales_in};
        tiles += (it.n + a.tile_elems - 1) / a.tile_elems;
        if (tiles > 0x7FFFFFFFull) return MQG_EINVAL;
    }
    a.tile_start[mqg::kMaxBatchTensors] = (uint32_t)tiles;
    const hipError_t err = mqg::launch_quantize_tensors(a, (uint32_t)tiles, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_aggregate_update_tensors(const mqg_update_item* items, uint32_t count, uint32_t W,
                                        uint32_t bits, uint32_t bucket, float lr, void* stream) {
    if (!valid_common(bits, bucket)) return MQG_EINVAL;
    mqg::BatchAggregateArgs a;
    uint32_t tiles = 0;
    const mqg_status st = update_batch_args(items, count, W, bits, bucket, lr, false, mqg::aggregate_batch_tile(), a, &tiles);
    if (st != MQG_OK || tiles == 0) return st;
    const hipError_t err = mqg::launch_aggregate_tensors(a, tiles, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_aggregate_update_minmax_tensors(const mqg_update_item* items, uint32_t count, uint32_t W,
                                               uint32_t bits, uint32_t bucket, float lr, void* stream) {
    const bool per_tensor = bucket == 0u;
    if (per_tensor ? (bits < 1u || bits > 8u) : !valid_common(bits, bucket)) return MQG_EINVAL;
    mqg::BatchAggregateArgs a;
    uint32_t tiles = 0;
    const mqg_status st = update_batch_args(items, count, W, bits, per_tensor ? 1024u : bucket, lr, true,
                                            mqg::aggregate_minmax_batch_tile(), a, &tiles);
    if (st != MQG_OK || tiles == 0) return st;
    a.per_tensor = per_tensor ? 1u : 0u;
    const hipError_t err = mqg::launch_aggregate_minmax_tensors(a, tiles, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_quantize_minmax_tensors(const mqg_quantize_item* items, uint32_t count, uint32_t bits, uint32_t bucket,
                                       void* stream) {
    const bool per_tensor = bucket == 0u;
    if (per_tensor ? (bits < 1u || bits > 8u) : !valid_common(bits, bucket)) return MQG_EINVAL;
    if (count > MQG_MAX_TENSORS) return MQG_EINVAL;
    if (count == 0) return MQG_OK;
    if (items == nullptr) return MQG_EINVAL;
    mqg::BatchQuantizeArgs a;
    a.common = mqg::QuantizeArgs{};
    a.common.bits = bits;
    a.common.bucket = per_tensor ? 1024u : bucket;      // a given range: the bucket only shapes the launch
    a.common.bucket_shift = log2_if_pow2(a.common.bucket);
    a.count = count;
    a.tile_elems = mqg::quantize_minmax_batch_tile(a.common.bucket, a.common.bucket_shift);
    mqg::TensorRangeBatch rb;
    uint64_t tiles = 0;
    for (uint32_t i = 0; i < mqg::kMaxBatchTensors; ++i) {
        a.tile_start[i] = (uint32_t)tiles;
        a.t[i] = mqg::BatchQuantizeArgs::Tensor{nullptr, 0, 0, nullptr, nullptr, nullptr};
        rb.grad[i] = nullptr;
        rb.n[i] = 0;
        rb.range[i] = nullptr;
        if (i >= count) continue;
        const mqg_quantize_item& it = items[i];
        if (it.scales_in != nullptr) return MQG_EINVAL;   // this encoder derives every range from the data
        if (it.n == 0) continue;
        if (it.grad == nullptr || it.packed_out == nullptr || it.scales_out == nullptr) return MQG_EINVAL;
        if (it.n > (UINT64_MAX >> 4)) return MQG_EINVAL;
        if (misaligned4(it.grad) || misaligned4(it.packed_out) || misaligned8(it.scales_out)) return MQG_EALIGN;
        if (per_tensor) {
            a.t[i] = mqg::BatchQuantizeArgs::Tensor{it.grad, it.n, 0, it.packed_out, nullptr, it.scales_out};
            rb.grad[i] = it.grad;
            rb.n[i] = it.n;
            rb.range[i] = it.scales_out;
        } else {
            a.t[i] = mqg::BatchQuantizeArgs::Tensor{it.grad, it.n, 0, it.packed_out, it.scales_out, nullptr};
        }
        tiles += (it.n + a.tile_elems - 1) / a.tile_elems;
        if (tiles > 0x7FFFFFFFull) return MQG_EINVAL;
    }
    a.tile_start[mqg::kMaxBatchTensors] = (uint32_t)tiles;
    if (tiles == 0) return MQG_OK;
    hipError_t err = hipSuccess;
    if (per_tensor) err = mqg::launch_tensor_range_batch(rb, count, static_cast<hipStream_t>(stream));
    if (err == hipSuccess) err = mqg::launch_quantize_minmax_tensors(a, (uint32_t)tiles, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_quantize_minmax(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket,
                               uint32_t* packed_out, float* ranges_out, void* stream) {
    if (!valid_common(bits, bucket)) return MQG_EINVAL;
    if (n == 0) return MQG_OK;
    if (grad == nullptr || packed_out == nullptr || ranges_out == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4)) return MQG_EINVAL;
    if (misaligned4(grad) || misaligned4(packed_out) || misaligned8(ranges_out)) return MQG_EALIGN;
    mqg::QuantizeArgs a = {};
    a.grad = grad;
    a.n = n;
    a.bits = bits;
    a.bucket = bucket;
    a.bucket_shift = log2_if_pow2(bucket);
    a.packed = packed_out;
    a.scales = ranges_out;
    const hipError_t err = mqg::launch_quantize_minmax(a, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_aggregate_update_minmax(const uint32_t* const* packed, const float* const* ranges, uint32_t W,
                                       uint64_t n, uint32_t bits, uint32_t bucket,
                                       float lr, float* params, void* stream) {
    if (!valid_common(bits, bucket)) return MQG_EINVAL;
    if (W < 1u || W > MQG_MAX_WORKERS) return MQG_EINVAL;
    if (n == 0) return MQG_OK;
    if (packed == nullptr || ranges == nullptr || params == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4)) return MQG_EINVAL;
    if (misaligned4(params)) return MQG_EALIGN;
    mqg::AggregateArgs a;
    a.stream_codes = 0u;
    const mqg_status tables = worker_tables(packed, ranges, W, true, a.packed, a.scales);
    if (tables != MQG_OK) return tables;
    a.W = W;
    a.n = n;
    a.bits = bits;
    a.bucket = bucket;
    a.bucket_shift = log2_if_pow2(bucket);
    a.neg_c = -(lr / (float)W);
    a.params = params;
    a.per_tensor = 0u;
    const hipError_t err = mqg::launch_aggregate_minmax(a, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_aggregate_requantize_minmax(const uint32_t* const* packed, const float* const* ranges, uint32_t W,
                                           uint64_t n, uint32_t bits, uint32_t bucket,
                                           uint32_t* packed_out, float* ranges_out, void* stream) {
    if (!valid_common(bits, bucket)) return MQG_EINVAL;
    if (W < 1u || W > MQG_MAX_WORKERS) return MQG_EINVAL;
    if (n == 0) return MQG_OK;
    if (packed == nullptr || ranges == nullptr || packed_out == nullptr || ranges_out == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4)) return MQG_EINVAL;
    if (misaligned4(packed_out) || misaligned8(ranges_out)) return MQG_EALIGN;
    mqg::RequantArgs ra = {};
    const mqg_status tables = worker_tables(packed, ranges, W, true, ra.packed, ra.scales);
    if (tables != MQG_OK) return tables;
    ra.W = W;
    ra.q.n = n;
    ra.q.bits = bits;
    ra.q.bucket = bucket;
    ra.q.bucket_shift = log2_if_pow2(bucket);
    ra.q.packed = packed_out;
    ra.q.scales = ranges_out;
    const hipError_t err = mqg::launch_requantize_minmax(ra, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_tensor_range(const float* grad, uint64_t n, float* range_out, void* stream) {
    if (n == 0) return MQG_OK;
    if (grad == nullptr || range_out == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4)) return MQG_EINVAL;
    if (misaligned4(grad) || misaligned8(range_out)) return MQG_EALIGN;
    const hipError_t err = mqg::launch_tensor_range(grad, n, range_out, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_quantize_minmax_tensor(const float* grad, uint64_t n, uint32_t bits,
                                      uint32_t* packed_out, float* range_out, void* stream) {
    if (bits < 1u || bits > 8u) return MQG_EINVAL;
    if (n == 0) return MQG_OK;
    if (grad == nullptr || packed_out == nullptr || range_out == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4)) return MQG_EINVAL;
    if (misaligned4(grad) || misaligned4(packed_out) || misaligned8(range_out)) return MQG_EALIGN;
    hipError_t err = mqg::launch_tensor_range(grad, n, range_out, static_cast<hipStream_t>(stream));
    if (err != hipSuccess) return MQG_ELAUNCH;
    mqg::QuantizeArgs a = {};
    a.grad = grad;
    a.n = n;
    a.bits = bits;
    a.bucket = 1024u;            // tiling only: every chunk takes the one range in scales_in
    a.bucket_shift = 10;
    a.scales_in = range_out;
    a.packed = packed_out;
    a.scales = nullptr;          // not written when the range is given
    err = mqg::launch_quantize_minmax(a, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_aggregate_update_minmax_tensor(const uint32_t* const* packed, const float* const* ranges,
                                              uint32_t W, uint64_t n, uint32_t bits,
                                              float lr, float* params, void* stream) {
    if (bits < 1u || bits > 8u) return MQG_EINVAL;
    if (W < 1u || W > MQG_MAX_WORKERS) return MQG_EINVAL;
    if (n == 0) return MQG_OK;
    if (packed == nullptr || ranges == nullptr || params == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4)) return MQG_EINVAL;
    if (misaligned4(params)) return MQG_EALIGN;
    mqg::AggregateArgs a;
    a.stream_codes = 0u;
    const mqg_status tables = worker_tables(packed, ranges, W, true, a.packed, a.scales);
    if (tables != MQG_OK) return tables;
    a.W = W;
    a.n = n;
    a.bits = bits;
    a.bucket = 1024u;            // tiling only: one (min, max) pair per worker
    a.bucket_shift = 10;
    a.neg_c = -(lr / (float)W);
    a.params = params;
    a.per_tensor = 1u;
    const hipError_t err = mqg::launch_aggregate_minmax(a, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_aggregate_requantize_minmax_tensor(const uint32_t* const* packed, const float* const* ranges,
                                                  uint32_t W, uint64_t n, uint32_t bits,
                                                  uint32_t* packed_out, float* range_out, void* stream) {
    if (bits < 1u || bits > 8u) return MQG_EINVAL;
    if (W < 1u || W > MQG_MAX_WORKERS) return MQG_EINVAL;
    if (n == 0) return MQG_OK;
    if (packed == nullptr || ranges == nullptr || packed_out == nullptr || range_out == nullptr) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4)) return MQG_EINVAL;
    if (misaligned4(packed_out) || misaligned8(range_out)) return MQG_EALIGN;
    mqg::RequantArgs ra = {};
    const mqg_status tables = worker_tables(packed, ranges, W, true, ra.packed, ra.scales);
    if (tables != MQG_OK) return tables;
    ra.W = W;
    ra.q.n = n;
    ra.q.bits = bits;
    ra.q.bucket = 1024u;            // tiling only: one range for the whole tensor
    ra.q.bucket_shift = 10;
    ra.q.packed = packed_out;
    ra.q.scales = range_out;
    const hipError_t err = mqg::launch_requantize_minmax_tensor(ra, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_sum_squares(const float* grad, uint64_t n, double* sumsq_out, void* stream) {
    if (sumsq_out == nullptr || (n > 0 && grad == nullptr)) return MQG_EINVAL;
    if (n > (UINT64_MAX >> 4)) return MQG_EINVAL;
    if ((n > 0 && misaligned4(grad)) || misaligned8(sumsq_out)) return MQG_EALIGN;
    const hipError_t err = mqg::launch_sum_squares(grad, n, sumsq_out, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

size_t mqg_sum_squares_workspace_bytes(uint32_t count) {
    return (size_t)count * mqg::sum_squares_batch_blocks() * sizeof(double);
}

mqg_status mqg_sum_squares_batch(const mqg_sumsq_item* items, uint32_t count, void* workspace, double* sumsq_out,
                                 void* stream) {
    if (count == 0u) return MQG_OK;
    if (workspace == nullptr) return MQG_EINVAL;
    mqg::SumSquaresBatch b;
    const mqg_status st = sumsq_batch_args(items, count, sumsq_out, b);
    if (st != MQG_OK) return st;
    if (misaligned8(workspace)) return MQG_EALIGN;
    const hipError_t err = mqg::launch_sum_squares_batch(b, count, static_cast<double*>(workspace), sumsq_out,
                                                         static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

mqg_status mqg_sum_squares_batch_static(const mqg_sumsq_item* items, uint32_t count, double* sumsq_out, void* stream) {
    if (count == 0u) return MQG_OK;
    mqg::SumSquaresBatch b;
    const mqg_status st = sumsq_batch_args(items, count, sumsq_out, b);   // count > MQG_MAX_SUMSQ_TENSORS: MQG_EINVAL
    if (st != MQG_OK) return st;
    const hipError_t err = mqg::launch_sum_squares_batch_static(b, count, sumsq_out, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? MQG_OK : MQG_ELAUNCH;
}

}  // extern "C"
