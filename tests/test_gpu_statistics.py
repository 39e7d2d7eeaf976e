"""Checks on the library's output alone (no oracle): laws the method must obey whatever the
implementation -- unbiased stochastic rounding, the step bound, convergence of quantized SGD with the
width chosen by the host agent."""
import math

import pytest
import torch

from paper_1804_08066_amd import mqgrad, workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("bits", [1, 2, 5])
def test_mean_over_iterations_approaches_the_gradient(bits):
    # params accumulate -dequantize(quantize(g)) with lr = 1, W = 1: after K iterations -params / K is
    # the mean de-quantized gradient; its deviation from g shrinks like (step / 2) / sqrt(K)
    n, bucket, K = 65536, 512, 1600
    g = workloads.normal(n, 0.01, 3, DEV)
    params = torch.zeros(n, device=DEV)
    pk, sc = mqgrad.alloc_outputs(n, bits, bucket, DEV)
    for it in range(K):
        mqgrad.mqg_quantize(g, bits, bucket, seed=11, iteration=it, packed_out=pk, scales_out=sc)
        mqgrad.mqg_aggregate_update([pk], [sc], n, bits, bucket, 1.0, params)
    torch.cuda.synchronize()
    mean = -params / K
    L = (1 << bits) - 1
    step = (2.0 * sc / L).repeat_interleave(bucket)[:n]
    dev = (mean - g).abs()
    # per element: standard deviation of the mean <= (step / 2) / sqrt(K); 6 sigma for 65 536 elements
    assert bool((dev <= 6.0 * 0.5 * step / math.sqrt(K) + 1e-6 * step).all())
    # and the deviations average out over elements as well (no systematic bias)
    assert abs(float(((mean - g) / step).mean())) < 4.0 * 0.5 / math.sqrt(K * n) + 2.0 ** -16


def test_single_quantization_stays_within_one_step():
    n, bucket = 100000 + 3, 256
    g = workloads.student_t(n, 3.0, 1e-3, 5, DEV)
    for bits in (1, 3, 8):
        pk, sc = mqgrad.mqg_quantize(g, bits, bucket, seed=2)
        params = torch.zeros(n, device=DEV)
        mqgrad.mqg_aggregate_update([pk], [sc], n, bits, bucket, 1.0, params)
        torch.cuda.synchronize()
        L = (1 << bits) - 1
        step = (2.0 * sc / L).repeat_interleave(bucket)[:n]
        assert bool(((-params - g).abs() <= step * (1 + 1e-5)).all())
        # the deterministic [min, max] encoder: within half a step
        pk2, rg = mqgrad.mqg_quantize_minmax(g, bits, bucket)
        p2 = torch.zeros(n, device=DEV)
        mqgrad.mqg_aggregate_update_minmax([pk2], [rg], n, bits, bucket, 1.0, p2)
        torch.cuda.synchronize()
        half = ((rg[1::2] - rg[0::2]) / L / 2).repeat_interleave(bucket)[:n]
        big = torch.maximum(rg[0::2].abs(), rg[1::2].abs()).repeat_interleave(bucket)[:n]
        assert bool(((-p2 - g).abs() <= half * (1 + 1e-5) + big * 2.0 ** -22).all())


def test_quantized_sgd_with_the_agent_choosing_the_width_converges():
    # minimise 0.5 |p - p*|^2 with W workers whose gradients carry independent noise; the host agent
    # (Algorithm 2) picks the width from the loss every few iterations, as in the paper's loop
    n, W, bucket, lr, iters = 200000, 4, 1024, 0.3, 120
    target = workloads.normal(n, 1.0, 1, DEV)
    params = torch.zeros(n, device=DEV)
    agent = mqgrad.Mdp(seed=3, bits_min=2, bits_max=8)
    outs = None
    bits = agent.current_bits
    losses, widths = [], []
    for it in range(iters):
        loss = 0.5 * float(((params - target) ** 2).mean())
        bits = agent.step(loss, 40.0 + 5.0 * bits)
        assert 2 <= bits <= 8
        grads = [(params - target) + workloads.normal(n, 0.05, 1000 * it + w, DEV) for w in range(W)]
        outs = [mqgrad.mqg_quantize(g, bits, bucket, seed=5, iteration=it, worker=w) for w, g in enumerate(grads)]
        mqgrad.mqg_aggregate_update([o[0] for o in outs], [o[1] for o in outs], n, bits, bucket, lr, params)
        losses.append(loss)
        widths.append(bits)
    torch.cuda.synchronize()
    assert losses[-1] < 1e-2 * losses[0]
    assert all(b2 >= b1 - 1 for b1, b2 in zip(widths, widths[1:]))        # an exploratory extra bit lasts one period
    agent.close()
