"""Pins for the oracle's deterministic min/max range-linear quantizer (the literal reading of the
Section 3.2 footnote: 2^K evenly spaced levels over the tensor's [min, max], nearest level) and for
the "Adaptive" baseline's bit rule of Section 4.1.  Each check ties the oracle to something other
than itself: closed forms, exact rational arithmetic, numpy library routines.  CPU only.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import policy_ref, ref
from exact_fp32 import f32_round

ALL_BITS = list(range(1, 9))


def rng(seed):
    return np.random.default_rng(seed)


# ---- ranges -------------------------------------------------------------------------------------

@pytest.mark.parametrize("n,bucket", [(1, 32), (31, 32), (1000, 96), (4096, 4096), (5000, 16384), (777, 64)])
def test_ranges_are_numpy_min_and_max_per_bucket(n, bucket):
    g = rng(n).normal(0, 1e-2, n).astype(np.float32)
    r = ref.minmax_ranges(g, bucket)
    nb = (n + bucket - 1) // bucket
    assert r.size == 2 * nb
    for k in range(nb):
        seg = g[k * bucket:(k + 1) * bucket]
        assert r[2 * k] == seg.min() and r[2 * k + 1] == seg.max()


def test_zero_bounds_are_stored_as_positive_zero():
    g = np.array([-0.0] * 32 + [0.0, -0.0] * 16 + [-0.0, -1.0] * 16 + [-0.0, 1.0] * 16, dtype=np.float32)
    r = ref.minmax_ranges(g, 32)
    assert r.view(np.uint32)[0] == 0 and r.view(np.uint32)[1] == 0
    assert r.view(np.uint32)[2] == 0 and r.view(np.uint32)[3] == 0
    assert r[4] == -1.0 and r.view(np.uint32)[5] == 0
    assert r.view(np.uint32)[6] == 0 and r[7] == 1.0


# ---- closed forms -------------------------------------------------------------------------------

@pytest.mark.parametrize("bits", ALL_BITS)
def test_integers_on_the_grid_are_their_own_codes(bits):
    # range [0, L]: the levels are the integers 0..L, so encode is the identity and decode is exact
    L = (1 << bits) - 1
    g = rng(bits).integers(0, L + 1, 4096).astype(np.float32)
    g[0], g[1] = 0.0, float(L)
    pk, r, codes = ref.quantize_minmax(g, bits, 4096, return_codes=True)
    assert r[0] == 0.0 and r[1] == float(L)
    assert np.array_equal(codes.astype(np.float32), g)
    assert np.array_equal(ref.dequantize_minmax(pk, r, g.size, bits, 4096), g)


@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("e,m0", [(-10, -3.0), (3, 40.0), (-20, 0.25)])
def test_shifted_power_of_two_grid_round_trips_exactly(bits, e, m0):
    # levels m0 + k * 2^e: range L * 2^e, every quantity in the encode and decode is exact
    L = (1 << bits) - 1
    k = rng(bits * 7 + e + 100).integers(0, L + 1, 2048)
    k[5], k[9] = 0, L
    g = (m0 + k * 2.0 ** e).astype(np.float32)
    assert np.array_equal(g.astype(np.float64), m0 + k * 2.0 ** e)      # representable
    pk, r, codes = ref.quantize_minmax(g, bits, 2048, return_codes=True)
    assert np.array_equal(codes, k.astype(np.uint8))
    assert np.array_equal(ref.dequantize_minmax(pk, r, g.size, bits, 2048), g)


@pytest.mark.parametrize("bits", ALL_BITS)
def test_ties_go_to_the_even_index(bits):
    L = (1 << bits) - 1
    for k in range(L):
        c = ref.nearest_code(k + 0.5, 0.0, float(L), bits)
        assert c == (k if k % 2 == 0 else k + 1), (bits, k, c)


def test_constant_and_tiny_ranges_have_one_level():
    g = np.full(100, 0.37, dtype=np.float32)
    for bits in ALL_BITS:
        pk, r, codes = ref.quantize_minmax(g, bits, 64, return_codes=True)
        assert not codes.any() and not pk.any()
        assert np.array_equal(ref.dequantize_minmax(pk, r, 100, bits, 64), g)
    tiny = np.array([0.0, 2.0 ** -100, 2.0 ** -99] * 11, dtype=np.float32)[:32]
    pk, r, codes = ref.quantize_minmax(tiny, 8, 32, return_codes=True)
    assert not codes.any()
    assert np.all(ref.dequantize_minmax(pk, r, 32, 8, 32) == 0.0)
    # just above the threshold the grid is live again
    wide = np.array([0.0, 2.0 ** -96] * 16, dtype=np.float32)
    _, _, codes = ref.quantize_minmax(wide, 8, 32, return_codes=True)
    assert codes.max() == 255


# ---- against exact arithmetic -------------------------------------------------------------------

@pytest.mark.parametrize("bits", ALL_BITS)
def test_code_is_the_nearest_level_in_exact_arithmetic(bits):
    # away from the mid-points between levels (by more than the fp32 rounding of the position) the
    # code must be THE nearest level of the exact grid mn + k (mx - mn) / L
    L = (1 << bits) - 1
    r = rng(100 + bits)
    checked = 0
    for _ in range(400):
        mn = np.float32(r.normal(0, 1e-2))
        mx = np.float32(mn + abs(r.normal(0, 2e-2)) + 1e-6)
        x = np.float32(mn + (mx - mn) * r.random())
        x = min(max(x, mn), mx)
        pos = (Fraction(float(x)) - Fraction(float(mn))) / (Fraction(float(mx)) - Fraction(float(mn))) * L
        near = math.floor(pos + Fraction(1, 2))
        if abs(pos - near) > Fraction(1, 2) - Fraction(L, 1 << 20):
            continue
        checked += 1
        assert ref.nearest_code(x, mn, mx, bits) == min(max(near, 0), L)
    assert checked > 300


@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("dist", ["normal", "uniform_pos", "outliers"])
def test_round_trip_error_is_at_most_half_a_step(bits, dist):
    r = rng(bits)
    n, bucket = 20000 + 17, 512
    if dist == "normal":
        g = r.normal(0, 1e-2, n)
    elif dist == "uniform_pos":
        g = r.uniform(0.5, 3.0, n)
    else:
        g = r.normal(0, 1e-3, n)
        g[::97] *= 50
    g = g.astype(np.float32)
    pk, rg = ref.quantize_minmax(g, bits, bucket)
    d = ref.dequantize_minmax(pk, rg, n, bits, bucket).astype(np.float64)
    L = (1 << bits) - 1
    k = np.arange(n) // bucket
    lo, hi = rg[0::2].astype(np.float64)[k], rg[1::2].astype(np.float64)[k]
    half = (hi - lo) / L / 2
    mag = np.maximum(np.abs(lo), np.abs(hi))
    assert np.all(np.abs(d - g) <= half * (1 + 1e-5) + mag * 2.0 ** -22)
    # and the bound is tight: a truncating encoder would reach a whole step
    assert np.max(np.abs(d - g) / half) > 0.9


@pytest.mark.parametrize("bits", ALL_BITS)
def test_extremes_take_the_end_codes_and_order_is_kept(bits):
    r = rng(bits + 50)
    g = r.normal(0.3, 1.0, 640).astype(np.float32)
    pk, rg, codes = ref.quantize_minmax(g, bits, 128, return_codes=True)
    L = (1 << bits) - 1
    d = ref.dequantize_minmax(pk, rg, 640, bits, 128)
    for k in range(5):
        seg, c = g[k * 128:(k + 1) * 128], codes[k * 128:(k + 1) * 128]
        assert c[seg.argmin()] == 0 and c[seg.argmax()] == L
        assert d[k * 128 + seg.argmin()] == seg.min()                      # level 0 is min exactly
        assert abs(float(d[k * 128 + seg.argmax()]) - float(seg.max())) <= 2.0 ** -22 * np.abs(seg).max()
        order = np.argsort(seg, kind="stable")
        assert np.all(np.diff(c[order].astype(int)) >= 0)                  # monotone


def test_values_outside_the_range_saturate():
    for bits in ALL_BITS:
        L = (1 << bits) - 1
        assert ref.nearest_code(5.0, -1.0, 2.0, bits) == L
        assert ref.nearest_code(1e30, -1.0, 2.0, bits) == L
        assert ref.nearest_code(-1.5, -1.0, 2.0, bits) == 0
        assert ref.nearest_code(-1e30, -1.0, 2.0, bits) == 0


@pytest.mark.parametrize("bits", [2, 5, 8])
def test_decode_is_one_division_and_one_fused_multiply_add(bits):
    # step = fl(fl(mx - mn) / L); value = fl(k * step + mn) with a single rounding
    L = (1 << bits) - 1
    r = rng(bits + 200)
    for _ in range(300):
        mn = np.float32(r.normal(0, 1e-2))
        mx = np.float32(mn + abs(r.normal(0, 2e-2)) + 1e-6)
        k = int(r.integers(0, L + 1))
        step = f32_round(f32_round(Fraction(float(mx)) - Fraction(float(mn))) / L)
        want = f32_round(k * step + Fraction(float(mn)))
        assert Fraction(float(ref.minmax_level_value(k, mn, mx, bits))) == want


@pytest.mark.parametrize("bits", [1, 3, 8])
def test_decode_matches_the_definition_in_fp64(bits):
    r = rng(bits + 70)
    n, bucket = 3000, 96
    g = r.normal(0, 1e-2, n).astype(np.float32)
    pk, rg, codes = ref.quantize_minmax(g, bits, bucket, return_codes=True)
    assert np.array_equal(ref.unpack(pk, n, bits), codes)
    L = (1 << bits) - 1
    k = np.arange(n) // bucket
    lo, hi = rg[0::2].astype(np.float64)[k], rg[1::2].astype(np.float64)[k]
    want = lo + codes.astype(np.float64) * (hi - lo) / L
    got = ref.dequantize_minmax(pk, rg, n, bits, bucket).astype(np.float64)
    assert np.all(np.abs(got - want) <= 2.0 ** -22 * np.maximum(np.abs(lo), np.abs(hi)))


def test_buckets_are_independent_and_the_tail_is_ragged():
    r = rng(9)
    g = r.normal(0, 1, 1000).astype(np.float32)
    pk, rg, codes = ref.quantize_minmax(g, 5, 96, return_codes=True)
    for k in range(11):
        seg = g[k * 96:(k + 1) * 96]
        _, rs, cs = ref.quantize_minmax(seg, 5, 96, return_codes=True)
        assert np.array_equal(rs, rg[2 * k:2 * k + 2]) and np.array_equal(cs, codes[k * 96:(k + 1) * 96])
    assert pk.size == (1000 * 5 + 31) // 32
    assert pk[-1] >> ((1000 * 5) % 32) == 0          # tail bits are zero


# ---- server step ----------------------------------------------------------------------------------

@pytest.mark.parametrize("W,bits", [(1, 4), (3, 2), (8, 8), (5, 5)])
def test_server_step_matches_the_mean_update_in_fp64(W, bits):
    r = rng(W * 10 + bits)
    n, bucket, lr = 5000, 256, 0.2
    grads = [r.normal(1e-3 * w, 1e-2, n).astype(np.float32) for w in range(W)]
    q = [ref.quantize_minmax(g, bits, bucket) for g in grads]
    p0 = r.uniform(-0.05, 0.05, n).astype(np.float32)
    p1 = ref.aggregate_update_minmax([x[0] for x in q], [x[1] for x in q], n, bits, bucket, lr, p0)
    deq = [ref.dequantize_minmax(x[0], x[1], n, bits, bucket).astype(np.float64) for x in q]
    want = p0.astype(np.float64) - float(np.float32(lr)) / W * sum(deq)
    mag = np.maximum(np.abs(p0), lr / W * sum(np.abs(d) for d in deq))
    assert np.all(np.abs(p1 - want) <= (W + 2) * 2.0 ** -24 * mag)
    # the mean of the de-quantized gradients is within half a step (averaged) of the true mean
    true = p0.astype(np.float64) - lr / W * sum(g.astype(np.float64) for g in grads)
    L = (1 << bits) - 1
    k = np.arange(n) // bucket
    half = sum((x[1][1::2].astype(np.float64) - x[1][0::2].astype(np.float64))[k] for x in q) / L / 2
    assert np.all(np.abs(p1 - true) <= lr / W * half * (1 + 1e-4) + 1e-7)


def test_server_step_with_one_worker_is_a_single_fused_update():
    r = rng(5)
    n = 2000
    g = r.normal(0, 1e-2, n).astype(np.float32)
    pk, rg = ref.quantize_minmax(g, 6, 128)
    p0 = r.uniform(-1, 1, n).astype(np.float32)
    p1 = ref.aggregate_update_minmax([pk], [rg], n, 6, 128, 0.3, p0)
    d = ref.dequantize_minmax(pk, rg, n, 6, 128)
    c = Fraction(float(np.float32(0.3)))
    for i in range(0, n, 5):
        assert Fraction(float(p1[i])) == f32_round(Fraction(float(p0[i])) - c * Fraction(float(d[i]))), i


# ---- the Adaptive baseline's rule ---------------------------------------------------------------

def test_adaptive_rule_thresholds():
    # K = 2 + floor(Z / 0.0005), kept inside 2..8: K = k exactly on [(k-2), (k-1)) * 0.0005
    assert policy_ref.adaptive_bits([0.0]) == 2
    assert policy_ref.adaptive_bits([0.0005]) == 3
    assert policy_ref.adaptive_bits([0.00049999]) == 2
    assert policy_ref.adaptive_bits([0.00149]) == 4
    assert policy_ref.adaptive_bits([0.003]) == 8
    assert policy_ref.adaptive_bits([0.0029]) == 7
    assert policy_ref.adaptive_bits([10.0]) == 8
    assert policy_ref.adaptive_bits([float("inf")]) == 8
    for i in range(2000):
        z = i * 2e-6
        want = min(8, 2 + int(Fraction(z) / Fraction(0.0005)))
        assert policy_ref.adaptive_bits([z]) == want


def test_adaptive_rule_uses_the_mean_over_workers_and_is_monotone():
    assert policy_ref.adaptive_bits([0.0, 0.002]) == policy_ref.adaptive_bits([0.001]) == 4
    assert policy_ref.adaptive_bits([0.0004, 0.0004, 0.0004, 0.0016]) == 3     # mean 0.0007
    prev = 0
    for i in range(500):
        k = policy_ref.adaptive_bits([i * 1e-5, i * 1.2e-5])
        assert k >= prev
        prev = k
    assert policy_ref.adaptive_bits([0.01], bits_min=1, bits_max=6) == 6
    assert policy_ref.adaptive_bits([0.0], base_bits=1, bits_min=1) == 1


def test_gradient_norm_is_numpy_norm():
    g = rng(3).normal(0, 1e-3, 10000).astype(np.float32)
    assert abs(policy_ref.gradient_norm(g) - np.linalg.norm(g.astype(np.float64))) <= 1e-12 * np.linalg.norm(g)
    assert policy_ref.gradient_norm(np.array([3.0, 4.0], dtype=np.float32)) == 5.0


# ---- full exchange with the [min, max] encoding ------------------------------------------------------

@pytest.mark.parametrize("whole_tensor", [False, True])
@pytest.mark.parametrize("W,bits", [(1, 3), (4, 2), (8, 8), (3, 5)])
def test_requantized_mean_is_within_half_a_step_of_the_mean(W, bits, whole_tensor):
    # whole_tensor: one bucket that covers the tensor -- Algorithm 1 as printed, one range per tensor
    r = rng(W * 13 + bits)
    n = 6000 + 5
    bucket = n if whole_tensor else 256
    grads = [r.normal(2e-3 * w, 1e-2, n).astype(np.float32) for w in range(W)]
    q = [ref.quantize_minmax(g, bits, bucket) for g in grads]
    deq = [ref.dequantize_minmax(x[0], x[1], n, bits, bucket).astype(np.float64) for x in q]
    s = ref.aggregate_sum_minmax([x[0] for x in q], [x[1] for x in q], n, bits, bucket)
    mag = sum(np.abs(d) for d in deq)
    assert np.all(np.abs(s - sum(deq)) <= W * 2.0 ** -24 * mag)            # fp32 chain against the fp64 sum
    pk, rg = ref.aggregate_requantize_minmax([x[0] for x in q], [x[1] for x in q], n, bits, bucket)
    # the stored range is [min, max] of the sum divided by W
    nb = (n + bucket - 1) // bucket
    for k in range(nb):
        seg = s[k * bucket:(k + 1) * bucket]
        assert rg[2 * k] == np.float32(seg.min()) / np.float32(W) and rg[2 * k + 1] == np.float32(seg.max()) / np.float32(W)
    # the codes are those of the sum over its own range
    pk_s, rg_s = ref.quantize_minmax(s, bits, bucket)
    assert np.array_equal(pk, pk_s)
    # and what the worker de-quantizes is the mean to within half a step (of the mean's grid)
    mean = sum(deq) / W
    got = ref.dequantize_minmax(pk, rg, n, bits, bucket).astype(np.float64)
    L = (1 << bits) - 1
    kk = np.arange(n) // bucket
    half = (rg[1::2].astype(np.float64) - rg[0::2].astype(np.float64))[kk] / L / 2
    big = np.maximum(np.abs(rg[0::2]), np.abs(rg[1::2])).astype(np.float64)[kk]
    assert np.all(np.abs(got - mean) <= half * (1 + 1e-4) + (W + 4) * 2.0 ** -23 * (big + mag / W))


def test_one_worker_on_the_grid_is_forwarded_unchanged():
    # W = 1: the sum is the de-quantized gradient, whose values are grid levels -- when the grid is exact
    # in fp32 (power-of-two step) re-encoding reproduces codes and range
    bits = 4
    k = rng(77).integers(0, 16, 4096)
    k[0], k[1] = 0, 15
    g = (-1.0 + k * 2.0 ** -6).astype(np.float32)
    pk, rg = ref.quantize_minmax(g, bits, 1024)
    pk2, rg2 = ref.aggregate_requantize_minmax([pk], [rg], g.size, bits, 1024)
    assert np.array_equal(pk, pk2) and np.array_equal(rg, rg2)
    p0 = rng(78).uniform(-1, 1, g.size).astype(np.float32)
    p1 = ref.aggregate_update_minmax([pk2], [rg2], g.size, bits, 1024, 0.25, p0)
    assert np.array_equal(p1, (p0.astype(np.float64) - 0.25 * g.astype(np.float64)).astype(np.float32))
