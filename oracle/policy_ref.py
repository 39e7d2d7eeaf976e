"""ORACLE (test infrastructure, not product code): the "Adaptive" baseline's bit rule.

Section 4.1 compares MQGrad with an adaptive method that sets the width from the size of the gradient:
the larger the gradient's norm, the more bits (Section 2, last paragraph on quantization).  The rule in
the paper's source is  K = 2 + Z / 0.0005  with Z the norm of the gradient to be quantized averaged over
the workers.  Readings: the quotient is truncated to an integer, and K is kept inside the range of
widths the system supports (2..8 in Section 4.1).
"""
import math


def gradient_norm(g):
    """L2 norm of one worker's gradient: square root of the exactly rounded sum of squares."""
    return math.sqrt(math.fsum(float(x) * float(x) for x in g))


def adaptive_bits(worker_norms, base_bits=2, norm_per_bit=0.0005, bits_min=2, bits_max=8):
    z = 0.0
    for v in worker_norms:
        z = z + float(v)
    z = z / len(worker_norms)
    k = base_bits + math.floor(z / norm_per_bit) if math.isfinite(z) else bits_max
    return int(min(max(k, bits_min), bits_max))
