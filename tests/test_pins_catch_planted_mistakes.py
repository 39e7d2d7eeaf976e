"""The pins are only worth something if a plausible mistake fails one of them.  One mistake at a time is
planted in a COPY of the oracle (wrong constant, swapped operand, dropped clamp, split fma, <= for <,
transposed bit order, sum for mean, wrong output index, ...), the copy is loaded in place of the oracle
(MQGRAD_ORACLE_LIB for the C++ library, MQGRAD_MDP_REF for the agent's reference), and the pin tests must
fail.  CPU only; nothing here touches the product library's arithmetic."""
import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_CPP = os.path.join(ROOT, "oracle", "mqgrad_oracle.cpp")
MDP_REF = os.path.join(ROOT, "oracle", "mdp_ref.py")

# (name, text in the oracle, what it is replaced by)
QUANTIZER_MISTAKES = [
 ("philox M0", "0xD2511F53u", "0xD2511F51u"),
 ("philox swap hi/lo", "const uint32_t n0 = hi1 ^ c1 ^ k0;", "const uint32_t n0 = hi0 ^ c1 ^ k0;"),
 ("philox 9 rounds", "round < 10", "round < 9"),
 ("key bump missing", "if (round > 0) { k0 += PHILOX_W0; k1 += PHILOX_W1; }", "if (round > 0) { k0 += PHILOX_W0; }"),
 ("group shift", "const uint64_t group = e >> 3;", "const uint64_t group = e >> 2;"),
 ("slot halves swapped", "return (slot & 1u) ? (word >> 16) : (word & 0xFFFFu);", "return (slot & 1u) ? (word & 0xFFFFu) : (word >> 16);"),
 ("counter order", "{(uint32_t)group, (uint32_t)(group >> 32), iteration, worker}", "{(uint32_t)group, (uint32_t)(group >> 32), worker, iteration}"),
 ("halfL wrong", "const float halfL = 0.5f * L;\n    const float a", "const float halfL = 0.5f * (L + 1.0f);\n    const float a"),
 ("no clamp", "u = std::fmin(std::fmax(u, 0.0f), L);", ""),
 ("r not centred", "((float)h + 0.5f) * 0x1p-16f", "((float)h) * 0x1p-16f"),
 ("r <= frac", "(r < frac) ? 1u : 0u", "(r <= frac) ? 1u : 0u"),
 ("round up inverted", "(r < frac) ? 1u : 0u", "(r > frac) ? 1u : 0u"),
 ("fma split", "float u = std::fmaf(x, a, halfL);", "float u = x * a + halfL;"),
 ("level sign", "return (float)(2 * (int)k - L) * d;", "return (float)(L - 2 * (int)k) * d;"),
 ("level offset", "return (float)(2 * (int)k - L) * d;", "return (float)(2 * (int)k - L - 1) * d;"),
 ("step uses L+1", "return s / L;\n}", "return s / (L + 1.0f);\n}"),
 ("max without abs", "const float a = std::fabs(g[i]);", "const float a = g[i];"),
 ("bucket off by one", "const uint64_t lo = k * bucket;", "const uint64_t lo = k * bucket + (k ? 1 : 0);"),
 ("pack big endian bits", "const uint32_t bit = (codes[i] >> t) & 1u;", "const uint32_t bit = (codes[i] >> (bits - 1 - t)) & 1u;"),
 ("pack word shift", "words[pos >> 5] |= bit << (pos & 31u);", "words[pos >> 5] |= bit << (31u - (pos & 31u));"),
 ("server sum not mean", "const float c = lr / (float)W;", "const float c = lr;"),
 ("server sign", "params[i] = std::fmaf(-c, acc, params[i]);", "params[i] = std::fmaf(c, acc, params[i]);"),
 ("server scale index", "const float d = scales[w][i / bucket] / (float)L;\n            acc = std::fmaf", "const float d = scales[w][0] / (float)L;\n            acc = std::fmaf"),
 ("server drops worker", "for (uint32_t w = 0; w < W; ++w) {\n            uint32_t k = 0;\n            for (uint32_t t = 0; t < bits; ++t) {\n                const uint64_t pos = i * bits + t;\n                k |= ((packed[w][pos >> 5] >> (pos & 31u)) & 1u) << t;\n            }\n            const float d = scales[w][i / bucket] / (float)L;", "for (uint32_t w = 0; w < W; ++w) {\n            uint32_t k = 0;\n            for (uint32_t t = 0; t < bits; ++t) {\n                const uint64_t pos = i * bits + t;\n                k |= ((packed[0][pos >> 5] >> (pos & 31u)) & 1u) << t;\n            }\n            const float d = scales[w][i / bucket] / (float)L;"),
 ("scale floor dropped", "if (!(s >= SCALE_FLOOR)) s = 0.0f;", ""),
 ("elem_base ignored", "uniform16(seed, iteration, worker, elem_base + i)", "uniform16(seed, iteration, worker, i)"),
 ("l2 without sqrt", "float s = (float)std::sqrt(acc);", "float s = (float)acc;"),
]

MINMAX_MISTAKES = [
 ("min/max swapped store", "ranges[2 * k] = mn;\n        ranges[2 * k + 1] = mx;", "ranges[2 * k] = mx;\n        ranges[2 * k + 1] = mn;"),
 ("min cmp", "if (g[i] < mn) mn = g[i];", "if (g[i] > mn) mn = g[i];"),
 ("range skips first", "float mn = g[lo_i], mx = g[lo_i];\n        for (uint64_t i = lo_i + 1;", "float mn = g[lo_i + (hi_i - lo_i > 1)], mx = mn;\n        for (uint64_t i = lo_i + 2;"),
 ("-0 kept", "if (mn == 0.0f) mn = 0.0f;   // -0 -> +0", ""),
 ("L is 2^b", "const float L = (float)((1u << bits) - 1u);\n    const float r = mx - mn;", "const float L = (float)(1u << bits);\n    const float r = mx - mn;"),
 ("floor not nearest", "float u = std::nearbyintf(d * a);", "float u = std::floor(d * a);"),
 ("half away", "float u = std::nearbyintf(d * a);", "float u = std::round(d * a);"),
 ("d not offset", "const float d = x - mn;", "const float d = x;"),
 ("threshold dropped", "const float a = (r >= 0x1p-96f) ? L / r : 0.0f;", "const float a = L / r;"),
 ("no upper clamp", "if (u > L) u = L;", ""),
 ("decode step L+1", "const float step = (mx - mn) / L;", "const float step = (mx - mn) / (L + 1.0f);"),
 ("decode from max", "return std::fmaf((float)k, step, mn);", "return std::fmaf(-(float)k, step, mx);"),
 ("decode no offset", "return std::fmaf((float)k, step, mn);", "return (float)k * step;"),
 ("decode split fma", "return std::fmaf((float)k, step, mn);", "return (float)k * step + mn;"),
 ("range index", "codes[i] = (uint8_t)orc_nearest_code(g[i], ranges[2 * k], ranges[2 * k + 1], bits);", "codes[i] = (uint8_t)orc_nearest_code(g[i], ranges[0], ranges[1], bits);"),
 ("deq range index", "out[i] = orc_minmax_level_value(codes[i], ranges[2 * k], ranges[2 * k + 1], bits);", "out[i] = orc_minmax_level_value(codes[i], ranges[0], ranges[1], bits);"),
 ("mm server sum not mean", "const float c = lr / (float)W;\n    for (uint64_t i = 0; i < n; ++i) params[i] = std::fmaf(-c, sum[i], params[i]);", "const float c = lr;\n    for (uint64_t i = 0; i < n; ++i) params[i] = std::fmaf(-c, sum[i], params[i]);"),
 ("mm server sign", "params[i] = std::fmaf(-c, sum[i], params[i]);", "params[i] = std::fmaf(c, sum[i], params[i]);"),
 ("mm server worker ranges", "orc_dequantize_minmax(packed[w], ranges[w], n, bits, bucket, v);", "orc_dequantize_minmax(packed[w], ranges[0], n, bits, bucket, v);"),
 ("mm server split fma", "params[i] = std::fmaf(-c, sum[i], params[i]);", "params[i] = params[i] - c * sum[i];"),
 ("mmx sum drops order", "for (uint64_t i = 0; i < n; ++i) sum[i] = sum[i] + v[i];\n    }\n    delete[] v;", "for (uint64_t i = 0; i < n; ++i) sum[i] = v[i];\n    }\n    delete[] v;"),
 ("mmx range not divided", "ranges_out[k] = ranges_out[k] / (float)W;", "ranges_out[k] = ranges_out[k];"),
 ("mmx range times W", "ranges_out[k] = ranges_out[k] / (float)W;", "ranges_out[k] = ranges_out[k] * (float)W;"),
 ("mmx quantizes worker 0", "orc_quantize_minmax(sum, n, bits, bucket, packed_out, ranges_out, nullptr);", "orc_dequantize_minmax(packed[0], ranges[0], n, bits, bucket, sum); orc_quantize_minmax(sum, n, bits, bucket, packed_out, ranges_out, nullptr);"),
]

MDP_MISTAKES = [
    ("moving average weights swapped", "prev = alpha * L + (1.0 - alpha) * prev", "prev = (1.0 - alpha) * L + alpha * prev"),
    ("slope against 0..T-1 with no intercept", "A = np.stack([i, np.ones(T)], axis=1)", "A = np.stack([i, np.zeros(T)], axis=1)"),
    ("reward sign", "return -(1.0 / cost_ms) * slope(smoothed) * gamma", "return (1.0 / cost_ms) * slope(smoothed) * gamma"),
    ("reward not divided by the cost", "return -(1.0 / cost_ms) * slope(smoothed) * gamma", "return -slope(smoothed) * gamma"),
    ("transition follows the taken action", "self.n_t = transition(n_prev, a_prev if self.follow_taken_action else greedy_prev)",
     "self.n_t = transition(n_prev, a_prev)"),
    ("greedy test inverted", "greedy = 1 if q[n - bits_min + 1] > q[n - bits_min] else 0", "greedy = 1 if q[n - bits_min + 1] < q[n - bits_min] else 0"),
    ("ties grow the width", "greedy = 1 if q[n - bits_min + 1] > q[n - bits_min] else 0", "greedy = 1 if q[n - bits_min + 1] >= q[n - bits_min] else 0"),
    ("exploration ignored", "return (1 - greedy if draw < epsilon else greedy), greedy", "return greedy, greedy"),
    ("maximum width not masked", "    if n >= bits_max:\n        return 0, 0\n", ""),
    ("Q(s, a) ignores the action", "o_prev = n_prev - self.bits_min + a_prev", "o_prev = n_prev - self.bits_min"),
    ("target ignores the action", "o_t = self.n_t - self.bits_min + a_t", "o_t = self.n_t - self.bits_min"),
    ("target uses the previous width", "o_t = self.n_t - self.bits_min + a_t", "o_t = n_prev - self.bits_min + a_t"),
    ("no discount", "td = r_prev + self.discount * q_t[o_t] - q_prev", "td = r_prev + q_t[o_t] - q_prev"),
    ("TD error sign", "td = r_prev + self.discount * q_t[o_t] - q_prev", "td = q_prev - r_prev - self.discount * q_t[o_t]"),
    ("gradient at the new state", "self.v = self.v + self.eta * td * q_gradient(self.v, self.shape, L_prev, o_prev)",
     "self.v = self.v + self.eta * td * q_gradient(self.v, self.shape, L_t, o_prev)"),
    ("step size dropped", "self.v = self.v + self.eta * td * q_gradient(", "self.v = self.v + td * q_gradient("),
    ("dead units pass gradient", "gb1[:] = W2[o] * (z > 0.0)", "gb1[:] = W2[o]"),
    ("hidden gradient from the wrong output", "gb1[:] = W2[o] * (z > 0.0)", "gb1[:] = W2[0] * (z > 0.0)"),
    ("W1 gradient transposed operand", "gW1[:, :] = np.outer(gb1, L)", "gW1[:, :] = np.outer(gb1, L[::-1])"),
    ("W2 gradient before the ReLU", "gW2[o, :] = np.maximum(z, 0.0)", "gW2[o, :] = z"),
    ("output bias not updated", "gb2[o] = 1.0", "gb2[o] = 0.0"),
    ("no ReLU in the forward pass", "return W2 @ np.maximum(W1 @ L + b1, 0.0) + b2", "return W2 @ (W1 @ L + b1) + b2"),
    ("sent width ignores the action", "self.bits_out = self.n_t + a_t", "self.bits_out = self.n_t"),
    ("inputs not normalised", "return np.array(self.window) / norm", "return np.array(self.window)"),
    ("decision every iteration", "if self.iteration % self.decide_every == 0:", "if True:"),
]


def run_pins(test_file, env_name, path):
    env = dict(os.environ)
    env[env_name] = path
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join("tests", test_file), "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    return r.returncode


def missed_cpp(mistakes, test_file):
    src = open(ORACLE_CPP).read()
    with tempfile.TemporaryDirectory() as tmp:
        def one(item):
            k, (name, old, new) = item
            assert src.count(old) >= 1, "the oracle no longer contains the text of mistake %r" % name
            cpp, so = os.path.join(tmp, "m%d.cpp" % k), os.path.join(tmp, "m%d.so" % k)
            with open(cpp, "w") as f:
                f.write(src.replace(old, new, 1))
            subprocess.check_call(["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared", cpp, "-o", so])
            return name if run_pins(test_file, "MQGRAD_ORACLE_LIB", so) == 0 else None
        with ThreadPoolExecutor(max_workers=6) as pool:
            return [m for m in pool.map(one, enumerate(mistakes)) if m]


def test_the_unchanged_oracle_passes_when_loaded_through_the_override():
    # the override itself must not be what makes the runs below fail
    from oracle import build as oracle_build
    assert run_pins("test_oracle_minmax_pins.py", "MQGRAD_ORACLE_LIB", oracle_build.build(force=False)) == 0
    assert run_pins("test_mdp.py", "MQGRAD_MDP_REF", MDP_REF) == 0


def test_every_planted_quantizer_mistake_fails_a_pin():
    assert missed_cpp(QUANTIZER_MISTAKES, "test_oracle_pins.py") == []


def test_every_planted_minmax_mistake_fails_a_pin():
    assert missed_cpp(MINMAX_MISTAKES, "test_oracle_minmax_pins.py") == []


def test_every_planted_agent_mistake_fails_a_pin():
    src = open(MDP_REF).read()
    with tempfile.TemporaryDirectory() as tmp:
        def one(item):
            k, (name, old, new) = item
            assert src.count(old) >= 1, "the reference no longer contains the text of mistake %r" % name
            path = os.path.join(tmp, "mdp_ref_m%d.py" % k)
            with open(path, "w") as f:
                f.write(src.replace(old, new, 1))
            return name if run_pins("test_mdp.py", "MQGRAD_MDP_REF", path) == 0 else None
        with ThreadPoolExecutor(max_workers=6) as pool:
            missed = [m for m in pool.map(one, enumerate(MDP_MISTAKES)) if m]
    assert missed == []
