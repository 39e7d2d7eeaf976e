"""Thin binding over the C-ABI library libmqgrad.so (see include/mqgrad.h).

Argument marshalling only: every step of the quantize / aggregate path runs in the library's
gfx950 kernels.  torch is used for device memory and streams.  There is no fallback: if the
library cannot be loaded, importing symbols from it raises.
"""
import ctypes as C
import os

import torch  # noqa: F401  (must be imported before the library so both share one HIP runtime)

from . import build as _build

MQG_OK, MQG_EINVAL, MQG_EALIGN, MQG_ELAUNCH = 0, -1, -2, -3
MQG_SCALE_MAXABS, MQG_SCALE_L2 = 0, 1
MQG_CODES_MAY_BE_CACHED, MQG_CODES_FROM_MEMORY = 0, 1
MQG_CODES_KEEP_CACHED, MQG_CODES_TO_MEMORY = 0, 1
MQG_MAX_WORKERS = 64

EXPORTS = [
    "mqg_status_string", "mqg_num_buckets", "mqg_packed_words",
    "mqg_quantize", "mqg_quantize_mode", "mqg_quantize_with_scales", "mqg_aggregate_update",
    "mqg_aggregate_requantize", "mqg_dequantize_update", "mqg_aggregate_mean", "mqg_quantize_tensors", "mqg_quantize_tensors_mode", "mqg_aggregate_update_tensors",
    "mqg_quantize_minmax", "mqg_aggregate_update_minmax", "mqg_aggregate_requantize_minmax",
    "mqg_tensor_range", "mqg_quantize_minmax_tensor", "mqg_aggregate_update_minmax_tensor", "mqg_aggregate_requantize_minmax_tensor", "mqg_sum_squares", "mqg_adaptive_default_config",
    "mqg_adaptive_bits",
    "mqg_mdp_default_config", "mqg_mdp_create", "mqg_mdp_destroy", "mqg_mdp_step", "mqg_mdp_step_workers",
    "mqg_mdp_current_bits", "mqg_mdp_smoothed_losses", "mqg_mdp_last_reward", "mqg_mdp_decisions",
    "mqg_mdp_num_weights", "mqg_mdp_get_weights", "mqg_mdp_set_weights", "mqg_mdp_q_values",
    "mqg_sum_squares_workspace_bytes", "mqg_sum_squares_batch", "mqg_sum_squares_batch_static",
    "mqg_quantize_minmax_tensors", "mqg_aggregate_update_minmax_tensors", "mqg_aggregate_requantize_mode",
    "mqg_aggregate_update_from", "mqg_quantize_to",
]


class MqgError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s" % (where, status_string(status)))


class MdpConfig(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("bits_min", C.c_uint32), ("bits_max", C.c_uint32),
                ("window", C.c_uint32), ("decide_every", C.c_uint32), ("hidden", C.c_uint32),
                ("alpha", C.c_double), ("epsilon", C.c_double), ("eta", C.c_double),
                ("reward_scale", C.c_double), ("discount", C.c_double), ("follow_taken_action", C.c_uint32)]


class AdaptiveConfig(C.Structure):
    _fields_ = [("base_bits", C.c_uint32), ("norm_per_bit", C.c_double), ("bits_min", C.c_uint32),
                ("bits_max", C.c_uint32)]


class SumsqItem(C.Structure):
    _fields_ = [("grad", C.c_void_p), ("n", C.c_uint64)]


class QuantizeItem(C.Structure):
    _fields_ = [("grad", C.c_void_p), ("n", C.c_uint64), ("elem_base", C.c_uint64),
                ("packed_out", C.c_void_p), ("scales_out", C.c_void_p), ("scales_in", C.c_void_p)]


class UpdateItem(C.Structure):
    _fields_ = [("n", C.c_uint64), ("params", C.c_void_p), ("packed", C.POINTER(C.c_void_p)),
                ("scales", C.POINTER(C.c_void_p)), ("raw", C.POINTER(C.c_void_p))]


MQG_MAX_TENSORS = 32
MQG_MAX_TENSOR_POINTERS = 256

_lib = None


def lib():
    """Load libmqgrad.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("MQGRAD_LIB")   # another build of the library (A/B timing of kernel variants)
    if path is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        elif _build.needs_build():
            import warnings
            warnings.warn("libmqgrad.so is older than its sources: run paper_1804_08066_amd/build.py (loading the stale library)")
    L = C.CDLL(path)
    vp, u32, u64, f32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_float
    L.mqg_status_string.argtypes = [C.c_int]
    L.mqg_status_string.restype = C.c_char_p
    L.mqg_num_buckets.argtypes = [u64, u32]
    L.mqg_num_buckets.restype = C.c_size_t
    L.mqg_packed_words.argtypes = [u64, u32]
    L.mqg_packed_words.restype = C.c_size_t
    L.mqg_quantize.argtypes = [vp, u64, u32, u32, u64, u32, u32, u64, vp, vp, vp]
    L.mqg_quantize.restype = C.c_int
    L.mqg_quantize_to.argtypes = [vp, u64, u32, u32, u64, u32, u32, u64, vp, vp, C.c_int, vp]
    L.mqg_quantize_to.restype = C.c_int
    L.mqg_quantize_mode.argtypes = [vp, u64, u32, u32, C.c_int, u64, u32, u32, u64, vp, vp, vp]
    L.mqg_quantize_mode.restype = C.c_int
    L.mqg_quantize_with_scales.argtypes = [vp, u64, u32, u32, u64, u32, u32, u64, vp, vp, vp, vp]
    L.mqg_quantize_with_scales.restype = C.c_int
    L.mqg_aggregate_update.argtypes = [C.POINTER(vp), C.POINTER(vp), u32, u64, u32, u32, f32, vp, vp]
    L.mqg_aggregate_update.restype = C.c_int
    L.mqg_aggregate_update_from.argtypes = [C.POINTER(vp), C.POINTER(vp), u32, u64, u32, u32, f32, vp, C.c_int, vp]
    L.mqg_aggregate_update_from.restype = C.c_int
    L.mqg_aggregate_requantize.argtypes = [C.POINTER(vp), C.POINTER(vp), u32, u64, u32, u32, u64, u32, u32, u64, vp, vp, vp]
    L.mqg_aggregate_requantize.restype = C.c_int
    L.mqg_aggregate_requantize_mode.argtypes = [C.POINTER(vp), C.POINTER(vp), u32, u64, u32, u32, C.c_int, u64, u32, u32, u64, vp, vp, vp]
    L.mqg_aggregate_requantize_mode.restype = C.c_int
    L.mqg_dequantize_update.argtypes = [vp, vp, u64, u32, u32, f32, vp, vp]
    L.mqg_dequantize_update.restype = C.c_int
    L.mqg_quantize_tensors.argtypes = [C.POINTER(QuantizeItem), u32, u32, u32, u64, u32, u32, vp]
    L.mqg_quantize_tensors.restype = C.c_int
    L.mqg_quantize_tensors_mode.argtypes = [C.POINTER(QuantizeItem), u32, u32, u32, C.c_int, u64, u32, u32, vp]
    L.mqg_quantize_tensors_mode.restype = C.c_int
    L.mqg_aggregate_update_tensors.argtypes = [C.POINTER(UpdateItem), u32, u32, u32, u32, f32, vp]
    L.mqg_aggregate_update_tensors.restype = C.c_int
    L.mqg_aggregate_update_minmax_tensors.argtypes = [C.POINTER(UpdateItem), u32, u32, u32, u32, f32, vp]
    L.mqg_aggregate_update_minmax_tensors.restype = C.c_int
    L.mqg_quantize_minmax_tensors.argtypes = [C.POINTER(QuantizeItem), u32, u32, u32, vp]
    L.mqg_quantize_minmax_tensors.restype = C.c_int
    L.mqg_quantize_minmax.argtypes = [vp, u64, u32, u32, vp, vp, vp]
    L.mqg_quantize_minmax.restype = C.c_int
    L.mqg_aggregate_update_minmax.argtypes = [C.POINTER(vp), C.POINTER(vp), u32, u64, u32, u32, f32, vp, vp]
    L.mqg_aggregate_update_minmax.restype = C.c_int
    L.mqg_aggregate_requantize_minmax.argtypes = [C.POINTER(vp), C.POINTER(vp), u32, u64, u32, u32, vp, vp, vp]
    L.mqg_aggregate_requantize_minmax.restype = C.c_int
    L.mqg_tensor_range.argtypes = [vp, u64, vp, vp]
    L.mqg_tensor_range.restype = C.c_int
    L.mqg_quantize_minmax_tensor.argtypes = [vp, u64, u32, vp, vp, vp]
    L.mqg_quantize_minmax_tensor.restype = C.c_int
    L.mqg_aggregate_update_minmax_tensor.argtypes = [C.POINTER(vp), C.POINTER(vp), u32, u64, u32, f32, vp, vp]
    L.mqg_aggregate_update_minmax_tensor.restype = C.c_int
    L.mqg_aggregate_requantize_minmax_tensor.argtypes = [C.POINTER(vp), C.POINTER(vp), u32, u64, u32, vp, vp, vp]
    L.mqg_aggregate_requantize_minmax_tensor.restype = C.c_int
    L.mqg_aggregate_mean.argtypes = [C.POINTER(vp), C.POINTER(vp), u32, u64, u32, u32, vp, vp]
    L.mqg_aggregate_mean.restype = C.c_int
    L.mqg_sum_squares.argtypes = [vp, u64, vp, vp]
    L.mqg_sum_squares.restype = C.c_int
    L.mqg_sum_squares_workspace_bytes.argtypes = [u32]
    L.mqg_sum_squares_workspace_bytes.restype = C.c_size_t
    L.mqg_sum_squares_batch.argtypes = [C.POINTER(SumsqItem), u32, vp, vp, vp]
    L.mqg_sum_squares_batch.restype = C.c_int
    L.mqg_sum_squares_batch_static.argtypes = [C.POINTER(SumsqItem), u32, vp, vp]
    L.mqg_sum_squares_batch_static.restype = C.c_int
    L.mqg_adaptive_default_config.argtypes = [C.POINTER(AdaptiveConfig)]
    L.mqg_adaptive_default_config.restype = None
    L.mqg_adaptive_bits.argtypes = [C.POINTER(C.c_double), u32, C.POINTER(AdaptiveConfig), C.POINTER(u32)]
    L.mqg_adaptive_bits.restype = C.c_int
    L.mqg_mdp_default_config.argtypes = [C.POINTER(MdpConfig)]
    L.mqg_mdp_default_config.restype = None
    L.mqg_mdp_create.argtypes = [C.POINTER(MdpConfig)]
    L.mqg_mdp_create.restype = vp
    L.mqg_mdp_destroy.argtypes = [vp]
    L.mqg_mdp_destroy.restype = None
    L.mqg_mdp_step.argtypes = [vp, C.c_double, C.c_double]
    L.mqg_mdp_step.restype = u32
    L.mqg_mdp_step_workers.argtypes = [vp, C.POINTER(C.c_double), u32, C.c_double]
    L.mqg_mdp_step_workers.restype = u32
    L.mqg_mdp_current_bits.argtypes = [vp]
    L.mqg_mdp_current_bits.restype = u32
    L.mqg_mdp_smoothed_losses.argtypes = [vp, C.POINTER(C.c_double)]
    L.mqg_mdp_smoothed_losses.restype = None
    L.mqg_mdp_last_reward.argtypes = [vp]
    L.mqg_mdp_last_reward.restype = C.c_double
    L.mqg_mdp_decisions.argtypes = [vp]
    L.mqg_mdp_decisions.restype = u64
    L.mqg_mdp_num_weights.argtypes = [vp]
    L.mqg_mdp_num_weights.restype = u32
    L.mqg_mdp_get_weights.argtypes = [vp, C.POINTER(C.c_double)]
    L.mqg_mdp_get_weights.restype = None
    L.mqg_mdp_set_weights.argtypes = [vp, C.POINTER(C.c_double)]
    L.mqg_mdp_set_weights.restype = None
    L.mqg_mdp_q_values.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.mqg_mdp_q_values.restype = None
    _lib = L
    return L


def status_string(status):
    return lib().mqg_status_string(int(status)).decode()


def mqg_num_buckets(n, bucket):
    return int(lib().mqg_num_buckets(n, bucket))


def mqg_packed_words(n, bits):
    return int(lib().mqg_packed_words(n, bits))


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(t, dtype, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (what, dtype))


def alloc_outputs(n, bits, bucket, device):
    packed = torch.empty(mqg_packed_words(n, bits), dtype=torch.int32, device=device)
    scales = torch.empty(mqg_num_buckets(n, bucket), dtype=torch.float32, device=device)
    return packed, scales


def mqg_quantize(grad, bits, bucket, seed, iteration=0, worker=0, elem_base=0,
                 packed_out=None, scales_out=None, stream=None, mode=None, scales_in=None, dest=None):
    """Worker side.  grad: fp32 CUDA tensor.  Returns (packed int32[words], scales fp32[nb]).

    mode selects mqg_quantize_mode; scales_in selects mqg_quantize_with_scales; dest (MQG_CODES_KEEP_CACHED /
    MQG_CODES_TO_MEMORY) selects mqg_quantize_to."""
    _check(grad, torch.float32, "grad")
    n = grad.numel()
    if packed_out is None or scales_out is None:
        p, s = alloc_outputs(n, bits, bucket, grad.device)
        packed_out = p if packed_out is None else packed_out
        scales_out = s if scales_out is None else scales_out
    _check(packed_out, torch.int32, "packed_out")
    _check(scales_out, torch.float32, "scales_out")
    if packed_out.numel() < mqg_packed_words(n, bits) or scales_out.numel() < mqg_num_buckets(n, bucket):
        raise ValueError("output buffers too small")
    L = lib()
    sh = _stream_handle(stream)
    if scales_in is not None:
        _check(scales_in, torch.float32, "scales_in")
        if scales_in.numel() < mqg_num_buckets(n, bucket):
            raise ValueError("scales_in too small")
        st = L.mqg_quantize_with_scales(grad.data_ptr(), n, bits, bucket, seed, iteration, worker,
                                        elem_base, scales_in.data_ptr(), packed_out.data_ptr(),
                                        scales_out.data_ptr(), sh)
    elif mode is not None:
        st = L.mqg_quantize_mode(grad.data_ptr(), n, bits, bucket, int(mode), seed, iteration, worker,
                                 elem_base, packed_out.data_ptr(), scales_out.data_ptr(), sh)
    elif dest is not None:
        st = L.mqg_quantize_to(grad.data_ptr(), n, bits, bucket, seed, iteration, worker, elem_base,
                               packed_out.data_ptr(), scales_out.data_ptr(), int(dest), sh)
    else:
        st = L.mqg_quantize(grad.data_ptr(), n, bits, bucket, seed, iteration, worker, elem_base,
                            packed_out.data_ptr(), scales_out.data_ptr(), sh)
    if st != MQG_OK:
        raise MqgError(st, "mqg_quantize")
    return packed_out, scales_out


def mqg_aggregate_update(packed, scales, n, bits, bucket, lr, params, stream=None, origin=MQG_CODES_MAY_BE_CACHED):
    """Server side.  packed / scales: lists of W CUDA tensors; params: fp32 CUDA tensor, updated in place.
    origin: MQG_CODES_FROM_MEMORY when the streams were not written by this GPU just before (same results,
    streaming loads of the code words at every width)."""
    W = len(packed)
    if W != len(scales):
        raise ValueError("packed and scales must have one entry per worker")
    _check(params, torch.float32, "params")
    if params.numel() != n:
        raise ValueError("params must have n elements")
    for p, s in zip(packed, scales):
        _check(p, torch.int32, "packed[w]")
        _check(s, torch.float32, "scales[w]")
        if p.numel() < mqg_packed_words(n, bits) or s.numel() < mqg_num_buckets(n, bucket):
            raise ValueError("a worker's buffers are too small for n")
    pa = (C.c_void_p * max(W, 1))(*[p.data_ptr() for p in packed])
    sa = (C.c_void_p * max(W, 1))(*[s.data_ptr() for s in scales])
    st = lib().mqg_aggregate_update_from(pa, sa, W, n, bits, bucket, lr, params.data_ptr(), int(origin), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_aggregate_update")
    return params


def _worker_arrays(packed, scales, n, bits, bucket):
    W = len(packed)
    if W != len(scales):
        raise ValueError("packed and scales must have one entry per worker")
    for p, s in zip(packed, scales):
        _check(p, torch.int32, "packed[w]")
        _check(s, torch.float32, "scales[w]")
        if p.numel() < mqg_packed_words(n, bits) or s.numel() < mqg_num_buckets(n, bucket):
            raise ValueError("a worker's buffers are too small for n")
    pa = (C.c_void_p * max(W, 1))(*[p.data_ptr() for p in packed])
    sa = (C.c_void_p * max(W, 1))(*[s.data_ptr() for s in scales])
    return W, pa, sa


def mqg_aggregate_mean(packed, scales, n, bits, bucket, mean_out=None, stream=None):
    """Mean over the workers of their de-quantized gradients (W = 1: De-quantize). Returns the fp32 tensor."""
    W, pa, sa = _worker_arrays(packed, scales, n, bits, bucket)
    if mean_out is None:
        mean_out = torch.empty(n, dtype=torch.float32, device=packed[0].device)
    _check(mean_out, torch.float32, "mean_out")
    if mean_out.numel() != n:
        raise ValueError("mean_out must have n elements")
    st = lib().mqg_aggregate_mean(pa, sa, W, n, bits, bucket, mean_out.data_ptr(), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_aggregate_mean")
    return mean_out


def mqg_aggregate_requantize(packed, scales, n, bits, bucket, seed, iteration=0, worker=0, elem_base=0,
                             packed_out=None, scales_out=None, stream=None, mode=MQG_SCALE_MAXABS):
    """Server's half of the full exchange: quantized mean of the W workers' gradients (mode: the bucket
    range of the sum, max-abs or L2 norm).  Returns (packed int32[words], scales fp32[nb])."""
    W, pa, sa = _worker_arrays(packed, scales, n, bits, bucket)
    dev = packed[0].device if W else "cuda"
    if packed_out is None or scales_out is None:
        p, s = alloc_outputs(n, bits, bucket, dev)
        packed_out = p if packed_out is None else packed_out
        scales_out = s if scales_out is None else scales_out
    _check(packed_out, torch.int32, "packed_out")
    _check(scales_out, torch.float32, "scales_out")
    if packed_out.numel() < mqg_packed_words(n, bits) or scales_out.numel() < mqg_num_buckets(n, bucket):
        raise ValueError("output buffers too small")
    st = lib().mqg_aggregate_requantize_mode(pa, sa, W, n, bits, bucket, int(mode), seed, iteration, worker, elem_base,
                                             packed_out.data_ptr(), scales_out.data_ptr(), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_aggregate_requantize")
    return packed_out, scales_out


def mqg_dequantize_update(packed, scales, n, bits, bucket, lr, params, stream=None):
    """Worker's half of the full exchange: params <- params - lr * De-quantize(packed, scales)."""
    _check(packed, torch.int32, "packed")
    _check(scales, torch.float32, "scales")
    _check(params, torch.float32, "params")
    if params.numel() != n or packed.numel() < mqg_packed_words(n, bits) or scales.numel() < mqg_num_buckets(n, bucket):
        raise ValueError("buffer sizes do not match n")
    st = lib().mqg_dequantize_update(packed.data_ptr(), scales.data_ptr(), n, bits, bucket, lr,
                                     params.data_ptr(), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_dequantize_update")
    return params


def mqg_quantize_tensors(grads, bits, bucket, seed, iteration=0, worker=0, elem_bases=None, outputs=None, stream=None,
                         scale_mode=MQG_SCALE_MAXABS, scales_in=None):
    """mqg_quantize for a list of layer tensors of one worker in one launch.
    scale_mode: the bucket range of the layers whose scales are computed; scales_in: optional list with, per
    layer, None or a float32 tensor of scales to use instead.  Returns a list of (packed, scales) per layer."""
    count = len(grads)
    if scales_in is None:
        scales_in = [None] * count
    if elem_bases is None:
        elem_bases = [0] * count
    if outputs is None:
        outputs = [alloc_outputs(g.numel(), bits, bucket, g.device) for g in grads]
    items = (QuantizeItem * max(count, 1))()
    for i, g in enumerate(grads):
        _check(g, torch.float32, "grads[%d]" % i)
        p, s = outputs[i]
        _check(p, torch.int32, "packed_out")
        _check(s, torch.float32, "scales_out")
        if p.numel() < mqg_packed_words(g.numel(), bits) or s.numel() < mqg_num_buckets(g.numel(), bucket):
            raise ValueError("output buffers too small")
        si = scales_in[i]
        if si is not None:
            _check(si, torch.float32, "scales_in")
            if si.numel() < mqg_num_buckets(g.numel(), bucket):
                raise ValueError("scales_in too small")
        items[i] = QuantizeItem(g.data_ptr(), g.numel(), elem_bases[i], p.data_ptr(), s.data_ptr(),
                                si.data_ptr() if si is not None else None)
    st = lib().mqg_quantize_tensors_mode(items, count, bits, bucket, int(scale_mode), seed, iteration, worker,
                                         _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_quantize_tensors")
    return outputs


def mqg_aggregate_update_tensors(layers, W, bits, bucket, lr, stream=None):
    """mqg_aggregate_update for a list of layers in one launch.

    Each layer is a dict with "params" and either ("packed": [W tensors], "scales": [W tensors]) for a
    quantized layer or "raw": [W fp32 gradient tensors] for a layer sent uncompressed."""
    items, keep = _update_items(layers, W, bits, bucket, 0)
    st = lib().mqg_aggregate_update_tensors(items, len(layers), W, bits, bucket, lr, _stream_handle(stream))
    del keep
    if st != MQG_OK:
        raise MqgError(st, "mqg_aggregate_update_tensors")


def _update_items(layers, W, bits, bucket, ranges):
    """The HOST table of a batched server step.  ranges: 0 = one scale per bucket, 1 = a (min, max) pair per
    bucket, 2 = one (min, max) pair per layer.  Returns (items, objects to keep alive during the call)."""
    count = len(layers)
    items = (UpdateItem * max(count, 1))()
    keep = []
    for i, layer in enumerate(layers):
        params = layer["params"]
        _check(params, torch.float32, "params")
        n = params.numel()
        if "raw" in layer:
            raw = layer["raw"]
            if len(raw) != W:
                raise ValueError("raw must have one gradient per worker")
            for g in raw:
                _check(g, torch.float32, "raw[w]")
                if g.numel() != n:
                    raise ValueError("raw gradient size differs from params")
            ra = (C.c_void_p * W)(*[g.data_ptr() for g in raw])
            keep.append(ra)
            items[i] = UpdateItem(n, params.data_ptr(), None, None, ra)
        else:
            packed, scales = layer["packed"], layer["scales"]
            if len(packed) != W or len(scales) != W:
                raise ValueError("packed/scales must have one entry per worker")
            need = mqg_num_buckets(n, bucket) if ranges == 0 else (2 * mqg_num_buckets(n, bucket) if ranges == 1 else 2)
            for pk, sc in zip(packed, scales):
                _check(pk, torch.int32, "packed[w]")
                _check(sc, torch.float32, "scales[w]")
                if pk.numel() < mqg_packed_words(n, bits) or sc.numel() < need:
                    raise ValueError("a worker's buffers are too small for n")
            pa = (C.c_void_p * W)(*[t.data_ptr() for t in packed])
            sa = (C.c_void_p * W)(*[t.data_ptr() for t in scales])
            keep.extend([pa, sa])
            items[i] = UpdateItem(n, params.data_ptr(), pa, sa, None)
    return items, keep


def mqg_quantize_minmax_tensors(grads, bits, bucket, outputs=None, stream=None):
    """mqg_quantize_minmax for a list of layer tensors in one launch; bucket = 0: one range per layer
    (mqg_quantize_minmax_tensor for every layer).  Returns a list of (packed, ranges) per layer."""
    count = len(grads)
    nr = (lambda n: 2 * mqg_num_buckets(n, bucket)) if bucket else (lambda n: 2)
    if outputs is None:
        outputs = [(torch.empty(mqg_packed_words(g.numel(), bits), dtype=torch.int32, device=g.device),
                    torch.empty(nr(g.numel()), dtype=torch.float32, device=g.device)) for g in grads]
    items = (QuantizeItem * max(count, 1))()
    for i, g in enumerate(grads):
        _check(g, torch.float32, "grads[%d]" % i)
        p, r = outputs[i]
        _check(p, torch.int32, "packed_out")
        _check(r, torch.float32, "ranges_out")
        if p.numel() < mqg_packed_words(g.numel(), bits) or r.numel() < nr(g.numel()):
            raise ValueError("output buffers too small")
        items[i] = QuantizeItem(g.data_ptr(), g.numel(), 0, p.data_ptr(), r.data_ptr(), None)
    st = lib().mqg_quantize_minmax_tensors(items, count, bits, bucket, _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_quantize_minmax_tensors")
    return outputs


def mqg_aggregate_update_minmax_tensors(layers, W, bits, bucket, lr, stream=None):
    """mqg_aggregate_update_minmax for a list of layers in one launch (bucket = 0: one (min, max) pair per worker
    and layer).  Layers as in mqg_aggregate_update_tensors, "scales" holding the range arrays."""
    items, keep = _update_items(layers, W, bits, bucket, 1 if bucket else 2)
    st = lib().mqg_aggregate_update_minmax_tensors(items, len(layers), W, bits, bucket, lr, _stream_handle(stream))
    del keep
    if st != MQG_OK:
        raise MqgError(st, "mqg_aggregate_update_minmax_tensors")


def mqg_quantize_minmax(grad, bits, bucket, packed_out=None, ranges_out=None, stream=None):
    """Deterministic [min, max] range-linear encode. Returns (packed int32 words, ranges fp32 (min, max) pairs)."""
    _check(grad, torch.float32, "grad")
    n = grad.numel()
    if packed_out is None:
        packed_out = torch.empty(mqg_packed_words(n, bits), dtype=torch.int32, device=grad.device)
    if ranges_out is None:
        ranges_out = torch.empty(2 * mqg_num_buckets(n, bucket), dtype=torch.float32, device=grad.device)
    _check(packed_out, torch.int32, "packed_out")
    _check(ranges_out, torch.float32, "ranges_out")
    if packed_out.numel() < mqg_packed_words(n, bits) or ranges_out.numel() < 2 * mqg_num_buckets(n, bucket):
        raise ValueError("output buffers too small")
    st = lib().mqg_quantize_minmax(grad.data_ptr(), n, bits, bucket, packed_out.data_ptr(), ranges_out.data_ptr(),
                                   _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_quantize_minmax")
    return packed_out, ranges_out


def mqg_aggregate_update_minmax(packed, ranges, n, bits, bucket, lr, params, stream=None):
    _check(params, torch.float32, "params")
    if params.numel() != n:
        raise ValueError("params must have n elements")
    W = len(packed)
    if W != len(ranges):
        raise ValueError("packed and ranges must have one entry per worker")
    for p, r in zip(packed, ranges):
        _check(p, torch.int32, "packed[w]")
        _check(r, torch.float32, "ranges[w]")
        if p.numel() < mqg_packed_words(n, bits) or r.numel() < 2 * mqg_num_buckets(n, bucket):
            raise ValueError("a worker's buffers are too small for n")
    pa = (C.c_void_p * max(W, 1))(*[p.data_ptr() for p in packed])
    ra = (C.c_void_p * max(W, 1))(*[r.data_ptr() for r in ranges])
    st = lib().mqg_aggregate_update_minmax(pa, ra, W, n, bits, bucket, lr, params.data_ptr(), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_aggregate_update_minmax")


def mqg_aggregate_requantize_minmax(packed, ranges, n, bits, bucket, packed_out=None, ranges_out=None, stream=None):
    """Server side of the full exchange with the [min, max] encoding. Returns (packed, ranges) of the mean."""
    W = len(packed)
    if W != len(ranges):
        raise ValueError("packed and ranges must have one entry per worker")
    for p, r in zip(packed, ranges):
        _check(p, torch.int32, "packed[w]")
        _check(r, torch.float32, "ranges[w]")
        if p.numel() < mqg_packed_words(n, bits) or r.numel() < 2 * mqg_num_buckets(n, bucket):
            raise ValueError("a worker's buffers are too small for n")
    dev = packed[0].device
    if packed_out is None:
        packed_out = torch.empty(mqg_packed_words(n, bits), dtype=torch.int32, device=dev)
    if ranges_out is None:
        ranges_out = torch.empty(2 * mqg_num_buckets(n, bucket), dtype=torch.float32, device=dev)
    _check(packed_out, torch.int32, "packed_out")
    _check(ranges_out, torch.float32, "ranges_out")
    if packed_out.numel() < mqg_packed_words(n, bits) or ranges_out.numel() < 2 * mqg_num_buckets(n, bucket):
        raise ValueError("output buffers too small")
    pa = (C.c_void_p * max(W, 1))(*[p.data_ptr() for p in packed])
    ra = (C.c_void_p * max(W, 1))(*[r.data_ptr() for r in ranges])
    st = lib().mqg_aggregate_requantize_minmax(pa, ra, W, n, bits, bucket, packed_out.data_ptr(),
                                               ranges_out.data_ptr(), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_aggregate_requantize_minmax")
    return packed_out, ranges_out


def mqg_tensor_range(grad, range_out=None, stream=None):
    """(min, max) of the whole tensor into a two-element float32 device tensor."""
    _check(grad, torch.float32, "grad")
    if range_out is None:
        range_out = torch.zeros(2, dtype=torch.float32, device=grad.device)
    _check(range_out, torch.float32, "range_out")
    st = lib().mqg_tensor_range(grad.data_ptr(), grad.numel(), range_out.data_ptr(), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_tensor_range")
    return range_out


def mqg_quantize_minmax_tensor(grad, bits, packed_out=None, range_out=None, stream=None):
    """The paper's encoder: one [min, max] for the whole tensor. Returns (packed, range)."""
    _check(grad, torch.float32, "grad")
    n = grad.numel()
    if packed_out is None:
        packed_out = torch.empty(mqg_packed_words(n, bits), dtype=torch.int32, device=grad.device)
    if range_out is None:
        range_out = torch.zeros(2, dtype=torch.float32, device=grad.device)
    _check(packed_out, torch.int32, "packed_out")
    _check(range_out, torch.float32, "range_out")
    if packed_out.numel() < mqg_packed_words(n, bits) or range_out.numel() < 2:
        raise ValueError("output buffers too small")
    st = lib().mqg_quantize_minmax_tensor(grad.data_ptr(), n, bits, packed_out.data_ptr(), range_out.data_ptr(),
                                          _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_quantize_minmax_tensor")
    return packed_out, range_out


def mqg_aggregate_update_minmax_tensor(packed, ranges, n, bits, lr, params, stream=None):
    _check(params, torch.float32, "params")
    if params.numel() != n:
        raise ValueError("params must have n elements")
    W = len(packed)
    if W != len(ranges):
        raise ValueError("packed and ranges must have one entry per worker")
    for p, r in zip(packed, ranges):
        _check(p, torch.int32, "packed[w]")
        _check(r, torch.float32, "ranges[w]")
        if p.numel() < mqg_packed_words(n, bits) or r.numel() < 2:
            raise ValueError("a worker's buffers are too small for n")
    pa = (C.c_void_p * max(W, 1))(*[p.data_ptr() for p in packed])
    ra = (C.c_void_p * max(W, 1))(*[r.data_ptr() for r in ranges])
    st = lib().mqg_aggregate_update_minmax_tensor(pa, ra, W, n, bits, lr, params.data_ptr(), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_aggregate_update_minmax_tensor")


def mqg_aggregate_requantize_minmax_tensor(packed, ranges, n, bits, packed_out=None, range_out=None, stream=None):
    """Server side of the full exchange with ONE [min, max] range per tensor. Returns (packed, range) of the mean."""
    W = len(packed)
    if W != len(ranges):
        raise ValueError("packed and ranges must have one entry per worker")
    for p, r in zip(packed, ranges):
        _check(p, torch.int32, "packed[w]")
        _check(r, torch.float32, "ranges[w]")
        if p.numel() < mqg_packed_words(n, bits) or r.numel() < 2:
            raise ValueError("a worker's buffers are too small for n")
    dev = packed[0].device
    if packed_out is None:
        packed_out = torch.empty(mqg_packed_words(n, bits), dtype=torch.int32, device=dev)
    if range_out is None:
        range_out = torch.zeros(2, dtype=torch.float32, device=dev)
    _check(packed_out, torch.int32, "packed_out")
    _check(range_out, torch.float32, "range_out")
    if packed_out.numel() < mqg_packed_words(n, bits) or range_out.numel() < 2:
        raise ValueError("output buffers too small")
    pa = (C.c_void_p * max(W, 1))(*[p.data_ptr() for p in packed])
    ra = (C.c_void_p * max(W, 1))(*[r.data_ptr() for r in ranges])
    st = lib().mqg_aggregate_requantize_minmax_tensor(pa, ra, W, n, bits, packed_out.data_ptr(), range_out.data_ptr(),
                                                      _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_aggregate_requantize_minmax_tensor")
    return packed_out, range_out


def mqg_sum_squares(grad, out=None, stream=None):
    """Sum of squares of a gradient in fp64, into a one-element float64 device tensor."""
    _check(grad, torch.float32, "grad")
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=grad.device)
    _check(out, torch.float64, "out")
    st = lib().mqg_sum_squares(grad.data_ptr(), grad.numel(), out.data_ptr(), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_sum_squares")
    return out


def mqg_sum_squares_workspace_bytes(count):
    return int(lib().mqg_sum_squares_workspace_bytes(int(count)))


def mqg_sum_squares_batch(grads, workspace=None, out=None, stream=None):
    """Sums of squares of several gradients in one call, each reproducible to the bit; returns a float64
    device tensor with one entry per gradient.  `workspace`: a device tensor of at least
    mqg_sum_squares_workspace_bytes(len(grads)) bytes (allocated here when not given)."""
    count = len(grads)
    for g in grads:
        _check(g, torch.float32, "grad")
    dev = grads[0].device if count else "cuda"
    if workspace is None:
        workspace = torch.empty(max(1, mqg_sum_squares_workspace_bytes(count) // 8), dtype=torch.float64, device=dev)
    if out is None:
        out = torch.empty(max(1, count), dtype=torch.float64, device=dev)[:count]
    _check(out, torch.float64, "out")
    items = (SumsqItem * max(1, count))()
    for k, g in enumerate(grads):
        items[k].grad = g.data_ptr()
        items[k].n = g.numel()
    st = lib().mqg_sum_squares_batch(items, count, workspace.data_ptr(), out.data_ptr(), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_sum_squares_batch")
    return out


def mqg_sum_squares_batch_static(grads, out, stream=None):
    """mqg_sum_squares_batch with the partial sums in the library's own device array: allocates nothing
    (`out`, a float64 device tensor with one entry per gradient, is the caller's)."""
    count = len(grads)
    for g in grads:
        _check(g, torch.float32, "grad")
    _check(out, torch.float64, "out")
    if out.numel() < count:
        raise ValueError("out holds fewer entries than there are gradients")
    items = (SumsqItem * max(1, count))()
    for k, g in enumerate(grads):
        items[k].grad = g.data_ptr()
        items[k].n = g.numel()
    st = lib().mqg_sum_squares_batch_static(items, count, out.data_ptr(), _stream_handle(stream))
    if st != MQG_OK:
        raise MqgError(st, "mqg_sum_squares_batch_static")
    return out


def mqg_adaptive_bits(worker_norms, **overrides):
    """Host only: the Adaptive baseline's width from the workers' gradient norms."""
    cfg = AdaptiveConfig()
    lib().mqg_adaptive_default_config(C.byref(cfg))
    for k, v in overrides.items():
        if not hasattr(cfg, k):
            raise TypeError("unknown adaptive option " + k)
        setattr(cfg, k, v)
    W = len(worker_norms)
    arr = (C.c_double * max(W, 1))(*[float(v) for v in worker_norms])
    out = C.c_uint32(0)
    st = lib().mqg_adaptive_bits(arr, W, C.byref(cfg), C.byref(out))
    if st != MQG_OK:
        raise MqgError(st, "mqg_adaptive_bits")
    return int(out.value)


class Mdp:
    """The host-side agent of Section 3.3 / Algorithm 2 (mqg_mdp_* of the C ABI)."""

    def __init__(self, **overrides):
        cfg = MdpConfig()
        lib().mqg_mdp_default_config(C.byref(cfg))
        for k, v in overrides.items():
            if not hasattr(cfg, k):
                raise AttributeError(k)
            setattr(cfg, k, v)
        self.cfg = cfg
        self._h = lib().mqg_mdp_create(C.byref(cfg))
        if not self._h:
            raise ValueError("mqg_mdp_create rejected the configuration")

    def step(self, loss, elapsed_ms):
        return int(lib().mqg_mdp_step(self._h, float(loss), float(elapsed_ms)))

    def step_workers(self, worker_losses, elapsed_ms):
        """Step with the mean of the workers' local losses (Algorithm 1, ReceiveLossThenSendbits)."""
        P = len(worker_losses)
        arr = (C.c_double * max(P, 1))(*[float(v) for v in worker_losses])
        return int(lib().mqg_mdp_step_workers(self._h, arr, P, float(elapsed_ms)))

    @property
    def current_bits(self):
        return int(lib().mqg_mdp_current_bits(self._h))

    @property
    def smoothed_losses(self):
        out = (C.c_double * self.cfg.window)()
        lib().mqg_mdp_smoothed_losses(self._h, out)
        return list(out)

    @property
    def last_reward(self):
        return float(lib().mqg_mdp_last_reward(self._h))

    @property
    def decisions(self):
        return int(lib().mqg_mdp_decisions(self._h))

    @property
    def weights(self):
        """The Q network's parameter vector [W1 | b1 | W2 | b2] as a list of floats."""
        out = (C.c_double * lib().mqg_mdp_num_weights(self._h))()
        lib().mqg_mdp_get_weights(self._h, out)
        return list(out)

    @weights.setter
    def weights(self, values):
        count = lib().mqg_mdp_num_weights(self._h)
        if len(values) != count:
            raise ValueError("expected %d weights" % count)
        lib().mqg_mdp_set_weights(self._h, (C.c_double * count)(*[float(v) for v in values]))

    def q_values(self, network_input):
        """One value per bit width for `window` inputs (smoothed losses divided by the first loss)."""
        if len(network_input) != self.cfg.window:
            raise ValueError("expected %d inputs" % self.cfg.window)
        out = (C.c_double * (self.cfg.bits_max - self.cfg.bits_min + 1))()
        lib().mqg_mdp_q_values(self._h, (C.c_double * self.cfg.window)(*[float(v) for v in network_input]), out)
        return list(out)

    def close(self):
        if self._h:
            lib().mqg_mdp_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
