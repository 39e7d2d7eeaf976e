"""Host checks of the arithmetic identities the server kernels' decode relies on (no GPU, no oracle).

The kernels never extract a code c as an integer.  They mask it in place at bit P of a word, OR in the
bits of 1.0f and apply one fma: with x = 1 + c * 2^(P - 23),
    fma(x, 2^(24 - P), -(2^(24 - P) + L)) == 2c - L            (L = 2^b - 1)
must hold exactly, for every width b, every code and both places P = 1 and P = 1 + b, and both constants
must be fp32 numbers whose bit patterns are the ones the kernels build with integer operations.
"""
import struct
from fractions import Fraction

import pytest

from exact_fp32 import f32_round


def bits_to_f32(u):
    return struct.unpack("<f", struct.pack("<I", u & 0xFFFFFFFF))[0]


@pytest.mark.parametrize("b", range(1, 9))
def test_mantissa_form_gives_the_centred_code_exactly(b):
    L = (1 << b) - 1
    for place, P in enumerate((1, 1 + b)):
        assert P + b <= 23                                   # the field stays inside the mantissa
        scale_bits = (150 - (P - 1)) << 23                   # 2^(24 - P), as the kernels build it
        minus_c_bits = 0x80000000 | scale_bits | (L << (P - 1))
        scale = Fraction(bits_to_f32(scale_bits))
        minus_c = Fraction(bits_to_f32(minus_c_bits))
        assert scale == Fraction(2) ** (24 - P)
        assert minus_c == -(Fraction(2) ** (24 - P) + L)
        field = L << P
        for c in range(L + 1):
            for junk in (0, 0xFFFFFFFF, 0xA5A5A5A5):         # the other bits of the word are arbitrary
                y = (junk & ~field & 0xFFFFFFFF) | (c << P)
                x = Fraction(bits_to_f32((y & field) | 0x3F800000))
                assert x == 1 + Fraction(c, 2 ** (23 - P))
                t = f32_round(x * scale + minus_c)           # one fma: a single rounding of the exact value
                assert t == 2 * c - L


@pytest.mark.parametrize("b", range(1, 9))
def test_rotations_put_a_quads_codes_at_the_two_places(b):
    """Widths that divide 32: rotating the word right by (sh - 1) mod 32 brings the quad's first code to
    bit 1; rotating that right by 2b brings the third there -- at 8 bits the fourth code wraps round the
    word, which is why the second step is a rotation and not a shift."""
    if 32 % b:
        pytest.skip("straddling widths take a funnel shift of two words instead")
    L = (1 << b) - 1
    rotr = lambda v, r: ((v >> (r & 31)) | (v << (32 - (r & 31)))) & 0xFFFFFFFF if r & 31 else v
    codes_per_word = 32 // b
    word = 0
    want = []
    for i in range(codes_per_word):
        c = (i * 7 + 3) & L
        want.append(c)
        word |= c << (i * b)
    for quad in range(codes_per_word // 4 if codes_per_word >= 4 else 0):
        sh = 4 * b * quad
        ya = rotr(word, (sh - 1) & 31)
        yb = rotr(ya, 2 * b)
        got = [(ya >> 1) & L, (ya >> (1 + b)) & L, (yb >> 1) & L, (yb >> (1 + b)) & L]
        assert got == want[4 * quad:4 * quad + 4]


@pytest.mark.parametrize("b", (3, 5, 6, 7))
def test_funnel_shift_form_for_straddling_widths(b):
    """A quad of 4b <= 28 bits taken from two words at bit offset sh (a multiple of 4): v << 1 holds codes
    0 and 1 at bits 1 and 1 + b, v >> (2b - 1) holds codes 2 and 3 there."""
    L = (1 << b) - 1
    stream = 0
    codes = [(i * 5 + 1) & L for i in range(64)]
    for i, c in enumerate(codes):
        stream |= c << (i * b)
    for quad in range(12):
        bit = 4 * b * quad
        lo = (stream >> (32 * (bit // 32))) & 0xFFFFFFFF
        hi = (stream >> (32 * (bit // 32 + 1))) & 0xFFFFFFFF
        sh = bit % 32
        v = (((hi << 32) | lo) >> sh) & 0xFFFFFFFF
        ya, yb = (v << 1) & 0xFFFFFFFF, v >> (2 * b - 1)
        got = [(ya >> 1) & L, (ya >> (1 + b)) & L, (yb >> 1) & L, (yb >> (1 + b)) & L]
        assert got == codes[4 * quad:4 * quad + 4]
