"""Shared helpers of the GPU parity tests: run the library on device tensors, the oracle on host copies."""
import numpy as np
import torch

from oracle import ref
from paper_1804_08066_amd import mqgrad


def to_u32(t):
    return t.detach().cpu().numpy().view(np.uint32)


def gpu_quantize(g, bits, bucket, seed, iteration=0, worker=0, elem_base=0, **kw):
    packed, scales = mqgrad.mqg_quantize(g, bits, bucket, seed, iteration, worker, elem_base, **kw)
    torch.cuda.synchronize()
    return to_u32(packed), scales.cpu().numpy()


def first_mismatch(a, b):
    idx = np.nonzero(a != b)[0]
    return None if idx.size == 0 else (int(idx[0]), int(idx.size))


def assert_quantize_parity(g, bits, bucket, seed, iteration=0, worker=0, elem_base=0, label=""):
    """Library vs oracle on the same tensor: scales and every packed word bit for bit."""
    gh = g.detach().cpu().numpy()
    pk_g, sc_g = gpu_quantize(g, bits, bucket, seed, iteration, worker, elem_base)
    pk_o, sc_o = ref.quantize(gh, bits, bucket, seed, iteration, worker, elem_base)
    assert sc_g.tobytes() == sc_o.tobytes(), "%s scales differ at %s" % (label, first_mismatch(sc_g.view(np.uint32), sc_o.view(np.uint32)))
    assert pk_g.shape == pk_o.shape
    assert np.array_equal(pk_g, pk_o), "%s packed words differ at %s" % (label, first_mismatch(pk_g, pk_o))
    return pk_o, sc_o


def param_tolerance(p_old, lr, W, dequantized):
    """1e-6 relative, with 'relative' taken against the largest of the magnitudes involved."""
    c = np.float32(lr) / np.float32(W)
    step = float(c) * sum(np.abs(d).astype(np.float64) for d in dequantized)
    return 1e-6 * np.maximum(np.abs(p_old).astype(np.float64), step)


def ulp_distance(a, b):
    ia = a.view(np.int32).astype(np.int64)
    ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, np.int64(-2 ** 31) - ia, ia)
    ib = np.where(ib < 0, np.int64(-2 ** 31) - ib, ib)
    return np.abs(ia - ib)
