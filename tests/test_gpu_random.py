"""Seeded random sweep over sizes, widths, bucket sizes, worker counts and alignments: every case is
compared with the oracle bit for bit (packed words, scales / ranges, updated parameters)."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_1804_08066_amd import mqgrad, workloads
from helpers import first_mismatch, to_u32, ulp_distance

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def cases(count, seed):
    r = np.random.default_rng(seed)
    out = []
    for i in range(count):
        n = int(np.exp(r.uniform(0, np.log(250000))))
        bits = int(r.integers(1, 9))
        if r.random() < 0.5:
            bucket = 32 << int(r.integers(0, 10))                  # power of two, 32 .. 16384
        else:
            bucket = 32 * int(r.integers(1, 513))                  # any multiple of 32
        W = int(r.integers(1, 10))
        out.append((i, n, bits, bucket, W, int(r.integers(0, 4)), int(r.integers(0, 4)), int(r.integers(0, 1 << 30))))
    return out


@pytest.mark.parametrize("case", cases(48, 2024), ids=lambda c: "n%d_b%d_B%d_W%d_o%d%d" % c[1:7])
def test_random_case_matches_oracle(case):
    i, n, bits, bucket, W, goff, poff, seed = case
    elem_base = 8 * (seed % 1000)
    grads = [workloads.normal_with_outliers(n + goff, 0.01, 0.01, 20.0, seed + w, DEV)[goff:] for w in range(W)]
    store = workloads.uniform(n + poff, -0.05, 0.05, seed + 99, DEV)
    lr = 0.05 + 0.01 * (seed % 7)

    # stochastic symmetric encoder
    params = store[poff:].clone() if poff == 0 else store[poff:]
    p0 = params.cpu().numpy().copy()
    q = [mqgrad.mqg_quantize(g, bits, bucket, seed=seed, iteration=i, worker=w, elem_base=elem_base)
         for w, g in enumerate(grads)]
    torch.cuda.synchronize()
    want = [ref.quantize(g.cpu().numpy(), bits, bucket, seed, i, w, elem_base) for w, g in enumerate(grads)]
    for w in range(W):
        assert q[w][1].cpu().numpy().tobytes() == want[w][1].tobytes(), "scales of worker %d" % w
        assert np.array_equal(to_u32(q[w][0]), want[w][0]), "worker %d: %s" % (w, first_mismatch(to_u32(q[w][0]), want[w][0]))
    mqgrad.mqg_aggregate_update([x[0] for x in q], [x[1] for x in q], n, bits, bucket, lr, params)
    torch.cuda.synchronize()
    p1 = ref.aggregate_update([x[0] for x in want], [x[1] for x in want], n, bits, bucket, lr, p0)
    assert ulp_distance(params.cpu().numpy(), p1).max() == 0

    # full exchange on the same streams
    mean_pk, mean_sc = mqgrad.mqg_aggregate_requantize([x[0] for x in q], [x[1] for x in q], n, bits, bucket,
                                                       seed=seed, iteration=i, worker=W, elem_base=elem_base)
    torch.cuda.synchronize()
    w_pk, w_sc = ref.aggregate_requantize([x[0] for x in want], [x[1] for x in want], n, bits, bucket, seed, i, W,
                                          elem_base)
    assert mean_sc.cpu().numpy().tobytes() == w_sc.tobytes()
    assert np.array_equal(to_u32(mean_pk), w_pk)

    # deterministic [min, max] encoder
    params2 = store[poff:]
    p0 = params2.cpu().numpy().copy()
    qm = [mqgrad.mqg_quantize_minmax(g, bits, bucket) for g in grads]
    torch.cuda.synchronize()
    wm = [ref.quantize_minmax(g.cpu().numpy(), bits, bucket) for g in grads]
    for w in range(W):
        assert qm[w][1].cpu().numpy().tobytes() == wm[w][1].tobytes(), "ranges of worker %d" % w
        assert np.array_equal(to_u32(qm[w][0]), wm[w][0])
    mpk, mrg = mqgrad.mqg_aggregate_requantize_minmax([x[0] for x in qm], [x[1] for x in qm], n, bits, bucket)
    torch.cuda.synchronize()
    w_pk, w_rg = ref.aggregate_requantize_minmax([x[0] for x in wm], [x[1] for x in wm], n, bits, bucket)
    assert mrg.cpu().numpy().tobytes() == w_rg.tobytes()
    assert np.array_equal(to_u32(mpk), w_pk)
    mqgrad.mqg_aggregate_update_minmax([x[0] for x in qm], [x[1] for x in qm], n, bits, bucket, lr, params2)
    torch.cuda.synchronize()
    p1 = ref.aggregate_update_minmax([x[0] for x in wm], [x[1] for x in wm], n, bits, bucket, lr, p0)
    assert ulp_distance(params2.cpu().numpy(), p1).max() == 0
