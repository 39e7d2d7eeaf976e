"""Seeded synthetic inputs shaped like the paper's workload.

The paper trains a CIFAR-10 CNN on a parameter server and quantizes the
gradients of its large fully connected layers (Section 4.1).  Neither the
dataset nor trained weights are used here: these generators produce fp32
tensors with the sizes, value distributions and structure named by the
benchmark configurations.  This module holds no part of the method's
arithmetic; it serves the oracle-side tests and the GPU-side tests alike.

Every generator takes a torch device; the same (seed, device) always gives
the same tensor.  Values differ between devices, so a parity test generates
once and hands the same tensor (copied to the host) to the oracle.
"""
import math

import torch

_CHUNK = 1 << 24  # generate large tensors in pieces to bound temporaries


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def normal(n, std, seed, device="cpu"):
    """n values ~ N(0, std^2)."""
    gen = _gen(seed, device)
    out = torch.empty(n, dtype=torch.float32, device=device)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        out[lo:hi].normal_(0.0, std, generator=gen)
    return out


def uniform(n, lo_v, hi_v, seed, device="cpu"):
    gen = _gen(seed, device)
    out = torch.empty(n, dtype=torch.float32, device=device)
    out.uniform_(lo_v, hi_v, generator=gen)
    return out


def laplace(n, scale, seed, device="cpu"):
    """n values ~ Laplace(0, scale), by inverting the CDF of a uniform draw."""
    gen = _gen(seed, device)
    u = torch.empty(n, dtype=torch.float32, device=device)
    u.uniform_(-0.5, 0.5, generator=gen)
    mag = torch.log1p(-2.0 * u.abs().clamp(max=0.5 - 1e-7))
    return (-scale) * torch.sign(u) * mag


def normal_with_outliers(n, std, outlier_prob, outlier_gain, seed, device="cpu"):
    """N(0, std^2) where a seeded Bernoulli(outlier_prob) subset is multiplied by outlier_gain."""
    gen = _gen(seed, device)
    out = torch.empty(n, dtype=torch.float32, device=device)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        part = out[lo:hi]
        part.normal_(0.0, std, generator=gen)
        mask = torch.empty(hi - lo, dtype=torch.float32, device=device)
        mask.uniform_(0.0, 1.0, generator=gen)
        part.mul_(torch.where(mask < outlier_prob, float(outlier_gain), 1.0))
    return out


def student_t(n, nu, scale, seed, device="cpu"):
    """scale * t_nu:  Z / sqrt(chi2_nu / nu) with integer nu, built from normal draws."""
    gen = _gen(seed, device)
    out = torch.empty(n, dtype=torch.float32, device=device)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        z = torch.empty(hi - lo, dtype=torch.float32, device=device).normal_(generator=gen)
        chi2 = torch.zeros(hi - lo, dtype=torch.float32, device=device)
        for _ in range(int(nu)):
            chi2 += torch.empty(hi - lo, dtype=torch.float32, device=device).normal_(generator=gen) ** 2
        out[lo:hi] = scale * z / torch.sqrt(chi2 / nu)
    return out


# ---- the benchmark configurations ------------------------------------------------

def config1(device="cpu"):
    """65,536 gradients ~ N(0, 0.01^2), seed 0; parameters ~ U(-0.05, 0.05); bucket 512; W=1; lr 0.1."""
    return {
        "grad": normal(65536, 0.01, 0, device),
        "params": uniform(65536, -0.05, 0.05, 1, device),
        "bucket": 512, "W": 1, "lr": 0.1, "bits": list(range(1, 9)),
    }


SMALL_CNN_SHAPES = [
    ("conv1.w", 5 * 5 * 3 * 64), ("conv1.b", 64),
    ("conv2.w", 5 * 5 * 64 * 64), ("conv2.b", 64),
    ("fc3.w", 2304 * 384), ("fc3.b", 384),
    ("fc4.w", 384 * 192), ("fc4.b", 192),
    ("fc5.w", 192 * 10), ("fc5.b", 10),
]


def config2_layer_scales(seed):
    """Per-layer Laplace scale s_l = 10^U(-4,-2), seeded (host side, a handful of numbers)."""
    gen = _gen(seed, "cpu")
    e = torch.empty(len(SMALL_CNN_SHAPES), dtype=torch.float64).uniform_(-4.0, -2.0, generator=gen)
    return [float(10.0 ** x) for x in e]


def config2_grads(iteration, worker, seed=0, device="cpu"):
    """One worker's gradients for one iteration: a list of fp32 layer tensors (~1.07M values)."""
    scales = config2_layer_scales(seed)
    out = []
    for li, ((_, n), s) in enumerate(zip(SMALL_CNN_SHAPES, scales)):
        out.append(laplace(n, s, 1000003 * (seed + 1) + 7919 * iteration + 101 * worker + li, device))
    return out


def config2_params(seed=0, device="cpu"):
    return [uniform(n, -0.05, 0.05, 555 + seed * 31 + li, device)
            for li, (_, n) in enumerate(SMALL_CNN_SHAPES)]


def config2_bits_sequence(iterations, seed=0):
    """Seeded per-iteration bit width over {1, 2, 4, 8}."""
    gen = _gen(seed + 77, "cpu")
    idx = torch.randint(0, 4, (iterations,), generator=gen)
    return [(1, 2, 4, 8)[int(i)] for i in idx]


def config2_elem_bases(bucket=512):
    """RNG stream offset of each layer: running sum of the layer sizes rounded up to the bucket."""
    bases, run = [], 0
    for _, n in SMALL_CNN_SHAPES:
        bases.append(run)
        run += (n + bucket - 1) // bucket * bucket
    return bases


def config3_grad(worker, n=25_600_000, device="cpu"):
    """ResNet-50-sized flat gradient ~ N(0, 1e-3^2) with 0.1% outliers at 100x."""
    return normal_with_outliers(n, 1e-3, 1e-3, 100.0, 3000 + worker, device)


def config4_grad(worker, n=100_000_000, device="cpu"):
    """Bandwidth-sweep gradient ~ N(0, 1e-2^2)."""
    return normal(n, 1e-2, 4000 + worker, device)


def config5_grad(worker, iteration, n=1_000_000_000, device="cpu"):
    """Large-model gradient ~ 1e-3 * Student-t(3)."""
    return student_t(n, 3, 1e-3, 5000 + 131 * iteration + worker, device)


def synthetic_loss_sequence(iterations, loss0=2.3, tau=8.0, noise_std=0.01, seed=0):
    """L_m = loss0 * exp(-m / tau) + N(0, noise_std^2): the loss stream fed to the host MDP."""
    gen = _gen(seed + 99, "cpu")
    noise = torch.empty(iterations, dtype=torch.float64).normal_(0.0, noise_std, generator=gen)
    return [loss0 * math.exp(-m / tau) + float(noise[m]) for m in range(iterations)]
