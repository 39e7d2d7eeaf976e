"""Parity at the edges of fp32: denormal and huge magnitudes, buckets at the 2^-96 threshold, zeros of
both signs, the far ends of every random-stream argument."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_1804_08066_amd import mqgrad, workloads
from helpers import first_mismatch, to_u32, ulp_distance

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def magnitudes(n, seed):
    """Buckets of 256 whose scale walks from denormals up to 1e37; signs and mantissas random."""
    g = workloads.normal(n, 1.0, seed, DEV)
    k = torch.arange(n, device=DEV) // 256
    expo = -149.0 + (k.double() * 7.3) % 272.0           # 2^-149 .. 2^123
    scale = torch.pow(torch.tensor(2.0, dtype=torch.float64, device=DEV), expo)
    out = (g.double() * scale).float()
    out[5::97] = 0.0
    out[6::97] = -0.0
    return out


@pytest.mark.parametrize("bits", [1, 2, 5, 8])
@pytest.mark.parametrize("bucket", [64, 96, 256, 1504, 4096])
def test_extreme_magnitudes_match_the_oracle(bits, bucket):
    n = 40 * 256 + 19
    grads = [magnitudes(n, 3 + w) for w in range(3)]
    assert all(bool(torch.isfinite(g).all()) for g in grads)
    q = [mqgrad.mqg_quantize(g, bits, bucket, seed=0xFEDCBA9876543210, iteration=0xFFFFFFFF, worker=0xFFFFFFFF - w,
                             elem_base=(1 << 40) + 8 * w) for w, g in enumerate(grads)]
    torch.cuda.synchronize()
    want = [ref.quantize(g.cpu().numpy(), bits, bucket, 0xFEDCBA9876543210, 0xFFFFFFFF, 0xFFFFFFFF - w,
                         (1 << 40) + 8 * w) for w, g in enumerate(grads)]
    for w in range(3):
        assert q[w][1].cpu().numpy().tobytes() == want[w][1].tobytes()
        assert np.array_equal(to_u32(q[w][0]), want[w][0]), first_mismatch(to_u32(q[w][0]), want[w][0])
    params = workloads.uniform(n, -1.0, 1.0, 9, DEV)
    p0 = params.cpu().numpy().copy()
    with np.errstate(over="ignore", invalid="ignore"):
        p1 = ref.aggregate_update([x[0] for x in want], [x[1] for x in want], n, bits, bucket, 1e-30, p0)
    mqgrad.mqg_aggregate_update([x[0] for x in q], [x[1] for x in q], n, bits, bucket, 1e-30, params)
    torch.cuda.synchronize()
    got = params.cpu().numpy()
    finite = np.isfinite(p1)
    assert finite.mean() > 0.9
    assert ulp_distance(got[finite], p1[finite]).max() == 0
    assert np.array_equal(np.isfinite(got), finite)


@pytest.mark.parametrize("bits", [1, 3, 8])
def test_extreme_magnitudes_minmax_encoder(bits):
    n = 40 * 256 + 19
    g = magnitudes(n, 11) * 0.25          # keeps max - min finite
    pk, rg = mqgrad.mqg_quantize_minmax(g, bits, 256)
    torch.cuda.synchronize()
    want_pk, want_rg = ref.quantize_minmax(g.cpu().numpy(), bits, 256)
    assert rg.cpu().numpy().tobytes() == want_rg.tobytes()
    assert np.array_equal(to_u32(pk), want_pk), first_mismatch(to_u32(pk), want_pk)


def test_scale_threshold_buckets():
    # buckets whose maximum sits just below, at and just above 2^-96, and all-zero / all-negative-zero ones
    vals = [2.0 ** -97, np.nextafter(np.float32(2.0 ** -96), np.float32(0)), 2.0 ** -96,
            np.nextafter(np.float32(2.0 ** -96), np.float32(1)), 0.0, -0.0, 2.0 ** -140]
    for bucket in (64, 96):   # the wave-local kernel and the cell-granular one
        g = torch.zeros(len(vals) * bucket, device=DEV)
        for i, v in enumerate(vals):
            g[i * bucket + 7] = float(v)
            g[i * bucket + 9] = -float(v) / 2
        for bits in (1, 4, 8):
            pk, sc = mqgrad.mqg_quantize(g, bits, bucket, seed=5)
            torch.cuda.synchronize()
            want_pk, want_sc = ref.quantize(g.cpu().numpy(), bits, bucket, 5)
            assert sc.cpu().numpy().tobytes() == want_sc.tobytes()
            assert np.array_equal(to_u32(pk), want_pk)
