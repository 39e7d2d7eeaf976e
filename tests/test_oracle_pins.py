"""Pins for the oracle: each check ties oracle/mqgrad_oracle.cpp to something other than itself --
published known-answer vectors, closed forms, exact rational arithmetic, numpy library routines,
brute force on tiny inputs, statistical laws.  CPU only.

The paper (MQGrad, arXiv 1804.08066) prints no worked numeric example of Quantize / De-quantize,
so there is no paper-printed value to store; what it fixes is the 2^K-level evenly spaced grid
(Section 3.2 footnote, Section 4.1), the server mean (Algorithm 1, ReceiveQGThenSendQG) and the
update rule (Algorithm 1, WorkerIterate).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from exact_fp32 import f32_round

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ALL_BITS = list(range(1, 9))


# ---- exact helpers (independent of the oracle) -------------------------------------------------

def exact_grid_position(x, s, bits):
    """u of the contract, with every fp32 rounding done in exact rational arithmetic."""
    L = (1 << bits) - 1
    halfL = Fraction(L, 2)
    a = f32_round(halfL / Fraction(float(s))) if s > 0 else Fraction(0)
    u = f32_round(Fraction(float(x)) * a + halfL)
    return min(max(u, Fraction(0)), Fraction(L))


# ---- Philox -------------------------------------------------------------------------------------

def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        out = ref.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_uniform16_slot_mapping():
    # element e: group e>>3 -> counter (lo, hi, iteration, worker); slot e&7 -> 16-bit half of word slot>>1
    seed, it, wk = 0x0123456789ABCDEF, 7, 3
    for e in [0, 1, 2, 7, 8, 9, 1023, (1 << 35) + 5, (1 << 35) + 6]:
        grp = e >> 3
        o = ref.philox4x32_10([grp & 0xFFFFFFFF, grp >> 32, it, wk], [seed & 0xFFFFFFFF, seed >> 32])
        word = int(o[(e & 7) >> 1])
        expect = (word >> 16) if (e & 1) else (word & 0xFFFF)
        assert ref.uniform16(seed, it, wk, e) == expect


def test_uniform16_chi_square_and_stream_independence():
    n = 1 << 17
    def stream(seed, it, wk):
        # through the quantizer's own path: codes at b=8 with x=0 are not informative, so call uniform16
        return np.array([ref.uniform16(seed, it, wk, e) for e in range(n)], dtype=np.float64)
    h00 = stream(11, 0, 0)
    counts = np.bincount((h00.astype(np.int64) >> 8), minlength=256)
    chi2 = ((counts - n / 256) ** 2 / (n / 256)).sum()
    assert chi2 < 255 + 6 * math.sqrt(2 * 255)          # ~6 sigma
    assert abs(h00.mean() - 32767.5) < 6 * 65536 / math.sqrt(12 * n)
    for other in (stream(11, 1, 0), stream(11, 0, 1), stream(12, 0, 0)):
        assert not np.array_equal(other, h00)
        c = np.corrcoef(h00, other)[0, 1]
        assert abs(c) < 5 / math.sqrt(n)


# ---- level grid ---------------------------------------------------------------------------------

@pytest.mark.parametrize("bits", ALL_BITS)
def test_level_set_closed_form(bits):
    # with s = L * 2^e every level is the integer (2k - L) * 2^e: 2^b values, symmetric, spacing 2^(e+1)
    L = (1 << bits) - 1
    for e in (-10, 0, 3):
        s = L * 2.0 ** e
        vals = [float(ref.level_value(k, s, bits)) for k in range(L + 1)]
        assert vals == [(2 * k - L) * 2.0 ** e for k in range(L + 1)]
        assert vals[0] == -s and vals[-1] == s
        assert all(v != 0 for v in vals)
        assert sorted(-v for v in vals) == vals


@pytest.mark.parametrize("bits", ALL_BITS)
def test_level_value_general_scale_is_evenly_spaced(bits):
    # general s: level(k) = s (2k-L)/L within 1 ulp of s (one division, one multiplication)
    L = (1 << bits) - 1
    for s in (0.0123, 1.0, 3.7e-5):
        s32 = np.float32(s)
        for k in range(L + 1):
            exact = Fraction(float(s32)) * (2 * k - L) / L
            got = Fraction(float(ref.level_value(k, s32, bits)))
            assert abs(got - exact) <= Fraction(float(np.spacing(s32)))


@pytest.mark.parametrize("bits", ALL_BITS)
def test_exact_round_trip_at_levels(bits):
    # inputs sitting exactly on levels come back unchanged for every seed
    L = (1 << bits) - 1
    e = -7
    bucket = 64
    ks = np.arange(2 * bucket) % (L + 1)
    ks[5] = L  # every bucket holds at least one element of magnitude s
    ks[bucket + 9] = 0
    g = ((2 * ks - L) * 2.0 ** e).astype(np.float32)
    for seed in (0, 1, 99):
        for it in (0, 5):
            packed, scales = ref.quantize(g, bits, bucket, seed, iteration=it, worker=2)
            assert np.all(scales == np.float32(L * 2.0 ** e))
            assert np.array_equal(ref.unpack(packed, g.size, bits), ks.astype(np.uint8))
            assert np.array_equal(ref.dequantize(packed, scales, g.size, bits, bucket), g)


# ---- stochastic rounding ------------------------------------------------------------------------

@pytest.mark.parametrize("bits", ALL_BITS)
def test_error_bound_every_element(bits):
    rng = np.random.default_rng(bits)
    bucket = 96
    g = np.concatenate([rng.normal(0, 0.01, 1000), rng.laplace(0, 1e-4, 1000), [0.0, 1e-30, -1e-30]]).astype(np.float32)
    L = (1 << bits) - 1
    for seed in range(3):
        packed, scales = ref.quantize(g, bits, bucket, seed)
        d = ref.dequantize(packed, scales, g.size, bits, bucket)
        s = np.repeat(scales, bucket)[: g.size].astype(np.float64)
        delta = 2 * s / L
        err = np.abs(d.astype(np.float64) - g.astype(np.float64))
        assert np.all(err < delta + 4 * np.spacing(s.astype(np.float32)))
        assert np.all(np.abs(d) <= s * (1 + 1e-6))


def test_rounding_is_unbiased_by_exhaustive_enumeration():
    # For fixed (x, s, b) enumerate all 65536 uniforms: the number that round up must be the count
    # of h with (h + 1/2)/65536 < frac, where frac comes from exact rational arithmetic.
    cases = [(0.0031, 0.0123, 3), (-0.0077, 0.0123, 2), (0.5, 1.0, 1), (-1.0, 1.0, 4), (1.0, 1.0, 8),
             (1e-5, 0.02, 8), (-0.019999, 0.02, 5), (3.3e-3, 7.7e-3, 7), (0.0, 0.5, 6), (2.5e-8, 1e-3, 1)]
    for x, s, bits in cases:
        x32, s32 = np.float32(x), np.float32(s)
        u = exact_grid_position(x32, s32, bits)
        lo = u.numerator // u.denominator
        frac = u - lo
        F = frac * 65536
        expect_up = 0 if F <= Fraction(1, 2) else min(65536, math.ceil(F - Fraction(1, 2)))
        codes = np.array([ref.round_code(x32, s32, bits, h) for h in range(65536)])
        assert set(np.unique(codes)) <= {lo, lo + 1}
        ups = int((codes == lo + 1).sum())
        assert ups == expect_up
        assert abs(Fraction(ups, 65536) - frac) <= Fraction(1, 1 << 17)
        # rounding up happens for the SMALL uniforms (r < frac)
        if 0 < ups < 65536:
            assert np.all(codes[:ups] == lo + 1) and np.all(codes[ups:] == lo)


def test_brute_force_tiny_vectors_textbook_rule():
    # exact-arithmetic inputs (s = L * 2^e, x on a 2^(e-6) lattice): the code must equal the textbook
    # "lower neighbour, or upper neighbour with probability equal to the relative position" rule,
    # evaluated in rationals, for a grid of uniforms.
    e = -4
    for bits in (1, 2, 3):
        L = (1 << bits) - 1
        s = Fraction(L) * Fraction(2) ** e
        lattice = [Fraction(j, 64) * Fraction(2) ** e for j in range(-64 * L, 64 * L + 1, 37)] + [s, -s]
        for xq in lattice:
            pos = (xq + s) / (2 * s) * L          # range-linear position in [0, L]
            lo = pos.numerator // pos.denominator
            frac = pos - lo
            for h in list(range(0, 65536, 4099)) + [65535]:
                r = Fraction(2 * h + 1, 1 << 17)
                expect = lo + (1 if r < frac else 0)
                assert ref.round_code(float(xq), float(s), bits, h) == expect


@pytest.mark.parametrize("bits", ALL_BITS)
def test_midpoint_uniform_gives_the_range_linear_encoder(bits):
    # h = 32767 makes r ~ 1/2: the quantizer degenerates to deterministic round-to-nearest, which is
    # the range-linear encode over [-s, s]:  q = round((x - min) / (max - min) * (2^K - 1)).
    rng = np.random.default_rng(100 + bits)
    L = (1 << bits) - 1
    s = np.float32(0.0371)
    x = rng.uniform(-float(s), float(s), 4000).astype(np.float32)
    pos = (x.astype(np.float64) + float(s)) / (2 * float(s)) * L
    keep = np.abs(pos - np.floor(pos) - 0.5) > 1e-4      # stay clear of ties
    q = np.floor(pos + 0.5).astype(np.int64)
    got = np.array([ref.round_code(v, s, bits, 32767) for v in x])
    assert np.array_equal(got[keep], q[keep])


def test_statistical_unbiasedness_and_variance_end_to_end():
    # includes Philox and the element->counter mapping: over many iterations the mean of the
    # de-quantized value converges to the input and its variance is (x - lo)(hi - x).
    rng = np.random.default_rng(5)
    n, bucket, iters = 256, 256, 3000
    g = rng.normal(0, 0.01, n).astype(np.float32)
    for bits in (1, 2, 4):
        L = (1 << bits) - 1
        acc = np.zeros(n)
        acc2 = np.zeros(n)
        for it in range(iters):
            packed, scales = ref.quantize(g, bits, bucket, 42, iteration=it, worker=1)
            d = ref.dequantize(packed, scales, n, bits, bucket).astype(np.float64)
            acc += d
            acc2 += d * d
        s = float(scales[0])
        delta = 2 * s / L
        mean = acc / iters
        var = acc2 / iters - mean ** 2
        x = g.astype(np.float64)
        assert np.all(np.abs(mean - x) < 5 * (delta / 2) / math.sqrt(iters))
        pos = (x + s) / delta
        lo = np.floor(pos)
        want_var = (pos - lo) * (1 - (pos - lo)) * delta ** 2
        assert abs(var.sum() - want_var.sum()) < 0.05 * want_var.sum()


# ---- scale --------------------------------------------------------------------------------------

def test_scale_is_numpy_maxabs_bit_for_bit():
    rng = np.random.default_rng(3)
    for n, bucket in [(4096, 512), (1000, 96), (33, 32), (1, 32), (5000, 16384)]:
        g = rng.laplace(0, 1e-3, n).astype(np.float32)
        sc = ref.bucket_scales(g, bucket)
        nb = (n + bucket - 1) // bucket
        want = np.array([np.max(np.abs(g[k * bucket:(k + 1) * bucket])) for k in range(nb)], dtype=np.float32)
        assert sc.tobytes() == want.tobytes()


def test_zero_and_tiny_buckets_contribute_exactly_zero():
    g = np.zeros(192, dtype=np.float32)
    g[64:128] = np.float32(2.0 ** -100)       # below the kept range
    g[128:] = 1.0
    for bits in ALL_BITS:
        packed, scales = ref.quantize(g, bits, 64, 9)
        assert scales[0] == 0 and scales[1] == 0 and scales[2] == 1
        d = ref.dequantize(packed, scales, g.size, bits, 64)
        assert np.all(d[:128] == 0)
        L = (1 << bits) - 1
        codes = ref.unpack(packed, g.size, bits)
        assert set(np.unique(codes[:128])) <= {L // 2, L // 2 + 1}   # coin flips between the middle codes
        assert np.all(codes[128:] == L)


def test_l2_scale_matches_numpy_norm():
    rng = np.random.default_rng(8)
    g = rng.normal(0, 0.01, 3000).astype(np.float32)
    sc = ref.bucket_scales(g, 512, ref.SCALE_L2)
    for k in range(sc.size):
        blk = g[k * 512:(k + 1) * 512].astype(np.float64)
        assert abs(float(sc[k]) - np.linalg.norm(blk)) <= 1e-7 * np.linalg.norm(blk)
        assert sc[k] >= np.max(np.abs(g[k * 512:(k + 1) * 512]))
    one = np.zeros(32, dtype=np.float32)
    one[3] = -0.3
    assert ref.bucket_scales(one, 32, ref.SCALE_L2)[0] == np.float32(0.3)


# ---- packing ------------------------------------------------------------------------------------

@pytest.mark.parametrize("bits", ALL_BITS)
def test_pack_unpack_identity_and_layout(bits):
    rng = np.random.default_rng(bits)
    for n in list(range(0, 70)) + [95, 96, 127, 128, 255, 300]:
        codes = rng.integers(0, 1 << bits, n, dtype=np.uint8)
        words = ref.pack(codes, bits)
        assert words.size == (n * bits + 31) // 32
        assert np.array_equal(ref.unpack(words, n, bits), codes)
        # numpy statement of the layout: bit t of code i is stream bit i*b + t, little-endian words
        bitmat = ((codes[:, None] >> np.arange(bits)) & 1).astype(np.uint8).reshape(-1)
        pad = (-bitmat.size) % 32
        stream = np.packbits(np.concatenate([bitmat, np.zeros(pad, np.uint8)]), bitorder="little")
        assert words.tobytes() == stream.tobytes()      # also proves the tail bits are zero


def test_pack_special_cases_are_library_routines():
    rng = np.random.default_rng(0)
    c1 = rng.integers(0, 2, 256, dtype=np.uint8)
    assert ref.pack(c1, 1).tobytes() == np.packbits(c1, bitorder="little").tobytes()
    c8 = rng.integers(0, 256, 256, dtype=np.uint8)
    assert ref.pack(c8, 8).tobytes() == c8.tobytes()
    c4 = rng.integers(0, 16, 256, dtype=np.uint8)
    assert ref.pack(c4, 4).tobytes() == (c4[0::2] | (c4[1::2] << 4)).astype(np.uint8).tobytes()


def test_code_msb_is_the_sign():
    g = np.array([-1.0, -0.4, -0.01, 0.01, 0.4, 1.0] + [0.0] * 26, dtype=np.float32)
    for bits in ALL_BITS:
        packed, scales = ref.quantize(g, bits, 32, 4)
        codes = ref.unpack(packed, g.size, bits)
        d = ref.dequantize(packed, scales, g.size, bits, 32)
        assert np.array_equal((codes >> (bits - 1)) & 1, (d > 0).astype(np.uint8))


# ---- server -------------------------------------------------------------------------------------

def _two_workers(n=3000, bits=5, bucket=96):
    rng = np.random.default_rng(17)
    gs = [rng.normal(0, 0.01, n).astype(np.float32) for _ in range(3)]
    qs = [ref.quantize(g, bits, bucket, 7, iteration=2, worker=w) for w, g in enumerate(gs)]
    p = rng.uniform(-0.05, 0.05, n).astype(np.float32)
    return gs, [q[0] for q in qs], [q[1] for q in qs], p


def test_server_special_cases():
    n, bits, bucket = 3000, 5, 96
    gs, pk, sc, p = _two_workers(n, bits, bucket)
    # lr = 0 leaves the parameters unchanged bit for bit
    assert ref.aggregate_update(pk[:1], sc[:1], n, bits, bucket, 0.0, p).tobytes() == p.tobytes()
    # W = 1, params = 0, lr = 1: the result is minus the de-quantized gradient
    out = ref.aggregate_update(pk[:1], sc[:1], n, bits, bucket, 1.0, np.zeros(n, np.float32))
    assert np.array_equal(out, -ref.dequantize(pk[0], sc[0], n, bits, bucket))
    # it is the MEAN over workers: W identical workers give the same step as one
    one = ref.aggregate_update(pk[:1], sc[:1], n, 5, bucket, 0.25, p)
    four = ref.aggregate_update([pk[0]] * 4, [sc[0]] * 4, n, bits, bucket, 0.25, p)
    mag = np.abs(p).astype(np.float64) + 0.25 * np.abs(ref.dequantize(pk[0], sc[0], n, bits, bucket))
    assert np.all(np.abs(one.astype(np.float64) - four) <= 4 * 2.0 ** -24 * mag)
    # direction: a positive gradient lowers the parameter
    d0 = ref.dequantize(pk[0], sc[0], n, bits, bucket)
    moved = ref.aggregate_update(pk[:1], sc[:1], n, bits, bucket, 0.5, p)
    assert np.all(np.sign(p.astype(np.float64) - moved) == np.sign(d0))


@pytest.mark.parametrize("bits", [1, 3, 8])
def test_server_matches_fp64_definition(bits):
    n, bucket, lr = 3000, 96, 0.1
    gs, pk, sc, p = _two_workers(n, bits, bucket)
    out = ref.aggregate_update(pk, sc, n, bits, bucket, lr, p).astype(np.float64)
    exact = ref.aggregate_update_f64(pk, sc, n, bits, bucket, float(np.float32(lr)), p)
    # and the fp64 definition itself against numpy on de-quantized vectors
    deq = [ref.dequantize(pk[w], sc[w], n, bits, bucket).astype(np.float64) for w in range(3)]
    plain = p.astype(np.float64) - float(np.float32(lr)) * (deq[0] + deq[1] + deq[2]) / 3
    mag = np.abs(p) + float(np.float32(lr)) * (np.abs(deq[0]) + np.abs(deq[1]) + np.abs(deq[2])) / 3
    assert np.all(np.abs(exact - plain) <= 1e-6 * mag)
    assert np.all(np.abs(out - exact) <= (3 + 2) * 2.0 ** -23 * mag)


def test_server_worker_order_changes_at_most_rounding():
    n, bits, bucket = 3000, 5, 96
    gs, pk, sc, p = _two_workers(n, bits, bucket)
    a = ref.aggregate_update(pk, sc, n, bits, bucket, 0.1, p)
    b = ref.aggregate_update(pk[::-1], sc[::-1], n, bits, bucket, 0.1, p)
    deq = sum(np.abs(ref.dequantize(pk[w], sc[w], n, bits, bucket)).astype(np.float64) for w in range(3))
    mag = np.abs(p).astype(np.float64) + 0.1 * deq / 3
    assert np.all(np.abs(a.astype(np.float64) - b) <= 3 * 2.0 ** -23 * mag)
    assert not np.array_equal(a, p)


def test_quantized_sgd_converges_at_8_bits_and_stalls_at_1_bit():
    rng = np.random.default_rng(2)
    n, bucket, W, lr = 2048, 512, 2, 0.5
    target = rng.normal(0, 1, n).astype(np.float32)
    final = {}
    for bits in (1, 8):
        p = np.zeros(n, dtype=np.float32)
        for it in range(40):
            grad = p - target                       # gradient of 0.5 * |p - target|^2
            qs = [ref.quantize(grad, bits, bucket, 3, iteration=it, worker=w) for w in range(W)]
            p = ref.aggregate_update([q[0] for q in qs], [q[1] for q in qs], n, bits, bucket, lr, p)
        final[bits] = float(np.abs(p - target).max())
    assert final[8] < 1e-6
    assert final[1] > 100 * final[8]


# ---- pins added after planting mistakes in a copy of the oracle ---------------------------------

def test_grid_position_is_a_single_rounding():
    # inputs for which rounding x*a first and then adding L/2 lands on a different fp32 than the
    # fused multiply-add: the count of up-rounding uniforms follows the fused value
    cases = [(0.5647523999214172, 0.6737864017486572, 8), (-0.36927440762519836, 0.5261039137840271, 7),
             (-0.475243479013443, 0.9990268349647522, 7), (0.08698460459709167, 0.09389900416135788, 7)]
    for x, s, bits in cases:
        x32, s32 = np.float32(x), np.float32(s)
        assert float(x32) == x and float(s32) == s
        L = (1 << bits) - 1
        a = f32_round(Fraction(L, 2) / Fraction(s))
        fused = f32_round(Fraction(x) * a + Fraction(L, 2))
        split = f32_round(f32_round(Fraction(x) * a) + Fraction(L, 2))
        assert fused != split
        lo = fused.numerator // fused.denominator
        F = (fused - lo) * 65536
        expect_up = 0 if F <= Fraction(1, 2) else min(65536, math.ceil(F - Fraction(1, 2)))
        codes = np.array([ref.round_code(x32, s32, bits, h) for h in range(0, 65536)])
        assert int((codes == lo + 1).sum()) == expect_up and set(np.unique(codes)) <= {lo, lo + 1}


@pytest.mark.parametrize("bits", ALL_BITS)
def test_values_beyond_the_scale_clamp_to_the_end_codes(bits):
    L = (1 << bits) - 1
    s = np.float32(0.37)
    for h in (0, 1, 32767, 65535):
        assert ref.round_code(2 * s, s, bits, h) == L
        assert ref.round_code(-2 * s, s, bits, h) == 0
        assert ref.round_code(np.float32(1e30), s, bits, h) == L
        assert ref.round_code(np.float32(-1e30), s, bits, h) == 0
    # and where fl((L/2)/s) * s exceeds L/2 the end elements themselves need the clamp
    found = 0
    for t in range(1, 4000):
        sc = np.float32(0.001 * t + 1e-4)
        a = f32_round(Fraction(L, 2) / Fraction(float(sc)))
        if a * Fraction(float(sc)) > Fraction(L, 2):
            found += 1
            for h in (0, 65535):
                assert ref.round_code(-sc, sc, bits, h) == 0 and ref.round_code(sc, sc, bits, h) == L
        if found >= 20:
            break
    assert found >= 1


def test_any_range_can_be_quantized_in_isolation():
    # the uniform of element i depends on elem_base + i only: quantizing a bucket-aligned tail with
    # elem_base = its first index reproduces the codes of the whole vector
    rng = np.random.default_rng(12)
    n, bucket = 4096 + 200, 256
    g = rng.normal(0, 0.01, n).astype(np.float32)
    for bits in (1, 3, 8):
        pk, sc = ref.quantize(g, bits, bucket, 99, iteration=4, worker=6, elem_base=1 << 33)
        whole = ref.unpack(pk, n, bits)
        for lo in (256, 1024, 4096):
            pk2, sc2 = ref.quantize(g[lo:], bits, bucket, 99, iteration=4, worker=6, elem_base=(1 << 33) + lo)
            assert np.array_equal(sc2, sc[lo // bucket:])
            assert np.array_equal(ref.unpack(pk2, n - lo, bits), whole[lo:])
        pk3, _ = ref.quantize(g, bits, bucket, 99, iteration=4, worker=6, elem_base=0)
        assert not np.array_equal(pk3, pk)


# ---- the full exchange: server sends the quantized mean back (Algorithm 1) ----------------------

def _workers(n, bits, bucket, W, seed=31):
    rng = np.random.default_rng(seed)
    gs = [rng.normal(0, 0.01 * (1 + w), n).astype(np.float32) for w in range(W)]
    qs = [ref.quantize(g, bits, bucket, 7, iteration=2, worker=w) for w, g in enumerate(gs)]
    return [q[0] for q in qs], [q[1] for q in qs]


@pytest.mark.parametrize("bits", [1, 3, 4, 8])
def test_aggregate_sum_matches_fp64_sum_of_dequantized(bits):
    n, bucket, W = 3000, 96, 5
    pk, sc = _workers(n, bits, bucket, W)
    got = ref.aggregate_sum(pk, sc, n, bits, bucket).astype(np.float64)
    deq = [ref.dequantize(pk[w], sc[w], n, bits, bucket).astype(np.float64) for w in range(W)]
    want = sum(deq)
    mag = sum(np.abs(d) for d in deq)
    assert np.all(np.abs(got - want) <= (W + 1) * 2.0 ** -23 * mag)
    assert np.array_equal(ref.aggregate_sum(pk[:1], sc[:1], n, bits, bucket), ref.dequantize(pk[0], sc[0], n, bits, bucket))


@pytest.mark.parametrize("bits", ALL_BITS)
def test_requantized_mean_is_within_one_step_of_the_mean(bits):
    n, bucket, W = 5000, 512, 4
    pk, sc = _workers(n, bits, bucket, W)
    L = (1 << bits) - 1
    mean = sum(ref.dequantize(pk[w], sc[w], n, bits, bucket).astype(np.float64) for w in range(W)) / W
    for seed in (0, 5):
        pk_m, sc_m = ref.aggregate_requantize(pk, sc, n, bits, bucket, seed, iteration=3, worker=W)
        # the stored range is max|sum| / W
        s_sum = ref.bucket_scales(ref.aggregate_sum(pk, sc, n, bits, bucket), bucket)
        assert np.array_equal(sc_m, s_sum / np.float32(W))
        back = ref.dequantize(pk_m, sc_m, n, bits, bucket).astype(np.float64)
        delta = 2 * np.repeat(sc_m, bucket)[:n].astype(np.float64) / L
        assert np.all(np.abs(back - mean) < delta * (1 + 1e-5) + 1e-12)
    # different seeds give different codes, same scales
    a = ref.aggregate_requantize(pk, sc, n, bits, bucket, 0, 3, W)
    b = ref.aggregate_requantize(pk, sc, n, bits, bucket, 1, 3, W)
    assert np.array_equal(a[1], b[1]) and (bits == 8 or not np.array_equal(a[0], b[0]))


@pytest.mark.parametrize("bits", ALL_BITS)
def test_requantizing_one_worker_on_exact_levels_is_the_identity(bits):
    # W = 1 and values on the grid of s = L * 2^e: the sum is exact, its range is s, every value sits on a level
    L = (1 << bits) - 1
    ks = (np.arange(256) * 7) % (L + 1)
    ks[0], ks[1] = 0, L
    g = ((2 * ks - L) * 2.0 ** -6).astype(np.float32)
    pk, sc = ref.quantize(g, bits, 128, 3)
    pk2, sc2 = ref.aggregate_requantize([pk], [sc], g.size, bits, 128, 99, 5, 1)
    assert np.array_equal(pk2, pk) and np.array_equal(sc2, sc)


def test_dequantize_update_special_cases_and_round_trip():
    n, bits, bucket, W, lr = 4000, 5, 256, 3, 0.25
    pk, sc = _workers(n, bits, bucket, W)
    rng = np.random.default_rng(1)
    p = rng.uniform(-0.05, 0.05, n).astype(np.float32)
    # params = 0, lr = 1: minus the de-quantized gradient; lr = 0: identity
    assert np.array_equal(ref.dequantize_update(pk[0], sc[0], n, bits, bucket, 1.0, np.zeros(n, np.float32)),
                          -ref.dequantize(pk[0], sc[0], n, bits, bucket))
    assert ref.dequantize_update(pk[0], sc[0], n, bits, bucket, 0.0, p).tobytes() == p.tobytes()
    # it is the W = 1 case of the server update
    assert np.array_equal(ref.dequantize_update(pk[1], sc[1], n, bits, bucket, lr, p),
                          ref.aggregate_update(pk[1:2], sc[1:2], n, bits, bucket, lr, p))
    # exchange end to end: worker update with the re-quantized mean stays within lr * step of the direct update
    pk_m, sc_m = ref.aggregate_requantize(pk, sc, n, bits, bucket, 4, 1, W)
    via_exchange = ref.dequantize_update(pk_m, sc_m, n, bits, bucket, lr, p).astype(np.float64)
    direct = ref.aggregate_update(pk, sc, n, bits, bucket, lr, p).astype(np.float64)
    delta = 2 * np.repeat(sc_m, bucket)[:n].astype(np.float64) / ((1 << bits) - 1)
    assert np.all(np.abs(via_exchange - direct) <= lr * delta * (1 + 1e-5) + 1e-9)
    assert np.abs(via_exchange - direct).max() > 0


def test_raw_layers_are_averaged_like_plain_sgd():
    rng = np.random.default_rng(4)
    n, W, lr = 1000, 5, 0.3
    gs = [rng.normal(0, 0.01, n).astype(np.float32) for _ in range(W)]
    p = rng.uniform(-0.05, 0.05, n).astype(np.float32)
    got = ref.average_update_raw(gs, lr, p).astype(np.float64)
    want = p.astype(np.float64) - float(np.float32(lr)) * np.mean(np.stack(gs).astype(np.float64), axis=0)
    mag = np.abs(p) + lr * np.mean(np.abs(np.stack(gs)), axis=0)
    assert np.all(np.abs(got - want) <= (W + 2) * 2.0 ** -23 * mag)
    assert np.array_equal(ref.average_update_raw(gs[:1], 1.0, np.zeros(n, np.float32)), -gs[0])
    assert ref.average_update_raw(gs, 0.0, p).tobytes() == p.tobytes()


# ---- the mean gradient as an output ---------------------------------------------------------------

@pytest.mark.parametrize("W,bits", [(1, 4), (3, 2), (8, 8), (7, 5)])
def test_mean_gradient_output(W, bits):
    rng = np.random.default_rng(W * 31 + bits)
    n, bucket = 4000 + 9, 256
    grads = [rng.normal(1e-3 * w, 1e-2, n).astype(np.float32) for w in range(W)]
    q = [ref.quantize(g, bits, bucket, 17, 2, w) for w, g in enumerate(grads)]
    mean = ref.aggregate_mean([x[0] for x in q], [x[1] for x in q], n, bits, bucket)
    deq = [ref.dequantize(x[0], x[1], n, bits, bucket).astype(np.float64) for x in q]
    want = sum(deq) / W
    mag = sum(np.abs(d) for d in deq) / W
    assert np.all(np.abs(mean - want) <= (W + 2) * 2.0 ** -24 * mag)
    if W == 1:
        assert np.array_equal(mean, ref.dequantize(q[0][0], q[0][1], n, bits, bucket))     # W = 1 is De-quantize
    # the division is a correctly rounded fp32 division of the fp32 sum
    s = ref.aggregate_sum([x[0] for x in q], [x[1] for x in q], n, bits, bucket)
    for i in range(0, n, 37):
        assert Fraction(float(mean[i])) == f32_round(Fraction(float(s[i])) / W)
    # consistency with the update: p - lr * mean agrees with the fused update to rounding
    p0 = rng.uniform(-0.05, 0.05, n).astype(np.float32)
    p1 = ref.aggregate_update([x[0] for x in q], [x[1] for x in q], n, bits, bucket, 0.1, p0)
    assert np.all(np.abs(p1 - (p0.astype(np.float64) - 0.1 * mean.astype(np.float64))) <= 4 * 2.0 ** -24 * np.maximum(np.abs(p0), 0.1 * mag))
