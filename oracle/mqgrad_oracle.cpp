// MQGrad hot-path ORACLE -- test infrastructure, not product code.
//
// A plain, slow, single-threaded CPU statement of what the gradient
// quantize / de-quantize / aggregate / update path computes.  It exists so
// that the GPU library can be checked against something that a reader can
// compare with the paper by eye.  Nothing in the product may call it: only
// tests, the smoke check and the benchmark's cpu_baseline leg do.  It shares
// no code with the GPU path.
//
// What the paper fixes (MQGrad, arXiv 1804.08066):
//   * Quantize(g, K) / De-quantize are a range-linear encode / decode to K
//     bits, i.e. 2^K evenly spaced levels over the tensor's range
//     (Section 3.2, footnote to the "quantize" step; Section 4.1 gives the
//     range of K as 2..8).
//   * The server de-quantizes every worker's gradient and takes the MEAN over
//     the P workers (Algorithm 1, function ReceiveQGThenSendQG; Section 3.1).
//   * The update is  w <- w - eta * g  (Algorithm 1, function WorkerIterate).
//   * One K is broadcast to all workers for an iteration (Algorithm 1,
//     function ReceiveLossThenSendbits).
// What the paper leaves open, and the reading taken here (each is listed in
// the design notes of the repository): symmetric range [-s, +s] with
// s = max|g| per bucket of `bucket` consecutive elements; stochastic rounding
// to the two neighbouring levels, driven by 16-bit uniforms from
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) keyed by the seed and
// counted by (element group, iteration, worker); codes packed little-endian
// into a dense stream of 32-bit words; bit widths 1..8.
//
// Arithmetic is fp32, round-to-nearest-even, denormals kept, no contraction
// (compile with -ffp-contract=off); the only fused operations are the
// explicit fmaf calls.

#include <cmath>
#include <cstdint>
#include <cstring>

namespace {

// ---- Philox4x32-10 (published algorithm; Salmon et al., SC'11) -----------
const uint32_t PHILOX_M0 = 0xD2511F53u;
const uint32_t PHILOX_M1 = 0xCD9E8D57u;
const uint32_t PHILOX_W0 = 0x9E3779B9u;  // golden ratio
const uint32_t PHILOX_W1 = 0xBB67AE85u;  // sqrt(3) - 1

void philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4]) {
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += PHILOX_W0; k1 += PHILOX_W1; }
        const uint64_t p0 = (uint64_t)PHILOX_M0 * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)PHILOX_M1 * (uint64_t)c2;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n1 = lo1;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        const uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// 16-bit uniform for global element index e.  One Philox call serves the 8
// consecutive elements of group e >> 3; element e takes 16-bit slot e & 7.
uint32_t uniform16(uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t e) {
    const uint64_t group = e >> 3;
    const uint32_t ctr[4] = {(uint32_t)group, (uint32_t)(group >> 32), iteration, worker};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t o[4];
    philox4x32_10(ctr, key, o);
    const uint32_t slot = (uint32_t)(e & 7u);
    const uint32_t word = o[slot >> 1];
    return (slot & 1u) ? (word >> 16) : (word & 0xFFFFu);
}

// ---- the level grid -------------------------------------------------------
// b bits, L = 2^b - 1.  The 2^b levels over the range [-s, +s] are
//   level(k) = s * (2k - L) / L ,  k = 0..L        (spacing 2s/L).
// L is odd, so the grid has no zero level and is symmetric: the top bit of k
// is the sign (1 = positive) and the low b-1 bits are the magnitude level
// (ones-complemented for negatives).

// Smallest bucket scale that is kept; below it the bucket is treated as all
// zero (keeps (L/2)/s finite for every b).
const float SCALE_FLOOR = 0x1p-96f;

float bucket_maxabs(const float* g, uint64_t count) {
    float s = 0.0f;
    for (uint64_t i = 0; i < count; ++i) {
        const float a = std::fabs(g[i]);
        if (a > s) s = a;
    }
    return s;
}

// sqrt of the fp64 sum of squares in index order, rounded once to fp32 and
// then bumped up to max|g| if rounding left it below (so |g_i| <= s holds).
float bucket_l2(const float* g, uint64_t count) {
    double acc = 0.0;
    for (uint64_t i = 0; i < count; ++i) acc += (double)g[i] * (double)g[i];
    float s = (float)std::sqrt(acc);
    const float m = bucket_maxabs(g, count);
    return (s < m) ? m : s;
}

// Stochastic rounding of one value x onto the code grid of (s, bits), given
// the 16-bit uniform h.  Returns the code k in 0..L.
uint32_t round_code(float x, float s, uint32_t bits, uint32_t h) {
    const float L = (float)((1u << bits) - 1u);
    const float halfL = 0.5f * L;
    const float a = (s > 0.0f) ? halfL / s : 0.0f;
    float u = std::fmaf(x, a, halfL);           // position on the grid, in [0, L]
    u = std::fmin(std::fmax(u, 0.0f), L);       // rounding may leave [0, L] by an ulp
    const float lo = std::floor(u);
    const float frac = u - lo;                  // exact, 0 <= frac < 1
    const float r = ((float)h + 0.5f) * 0x1p-16f;  // exact, in (0, 1)
    return (uint32_t)lo + ((r < frac) ? 1u : 0u);
}

float dequant_step(float s, uint32_t bits) {
    const float L = (float)((1u << bits) - 1u);
    return s / L;
}

float dequant_value(uint32_t k, float d, uint32_t bits) {
    const int L = (int)((1u << bits) - 1u);
    return (float)(2 * (int)k - L) * d;
}

}  // namespace

extern "C" {

void orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    philox4x32_10(ctr, key, out);
}

uint32_t orc_uniform16(uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t e) {
    return uniform16(seed, iteration, worker, e);
}

uint64_t orc_num_buckets(uint64_t n, uint32_t bucket) { return (n + bucket - 1) / bucket; }

uint64_t orc_packed_words(uint64_t n, uint32_t bits) { return (n * bits + 31) / 32; }

// scale_mode 0: max-abs, 1: L2 norm.  Scales below 2^-96 are stored as 0.
void orc_bucket_scales(const float* g, uint64_t n, uint32_t bucket, int scale_mode, float* scales) {
    const uint64_t nb = orc_num_buckets(n, bucket);
    for (uint64_t k = 0; k < nb; ++k) {
        const uint64_t lo = k * bucket;
        const uint64_t cnt = (n - lo < bucket) ? (n - lo) : bucket;
        float s = (scale_mode == 1) ? bucket_l2(g + lo, cnt) : bucket_maxabs(g + lo, cnt);
        if (!(s >= SCALE_FLOOR)) s = 0.0f;
        scales[k] = s;
    }
}

uint32_t orc_round_code(float x, float s, uint32_t bits, uint32_t h) {
    return round_code(x, s, bits, h);
}

// value of code k on the grid of scale s (what the server reconstructs)
float orc_level_value(uint32_t k, float s, uint32_t bits) {
    return dequant_value(k, dequant_step(s, bits), bits);
}

// Codes (one byte each) for a gradient, using the given per-bucket scales.
void orc_quantize_codes(const float* g, uint64_t n, uint32_t bits, uint32_t bucket,
                        uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                        const float* scales, uint8_t* codes) {
    for (uint64_t i = 0; i < n; ++i) {
        const float s = scales[i / bucket];
        const uint32_t h = uniform16(seed, iteration, worker, elem_base + i);
        codes[i] = (uint8_t)round_code(g[i], s, bits, h);
    }
}

// Dense little-endian bit stream: code i occupies stream bits [i*b, i*b+b),
// least significant code bit first; unused tail bits of the last word are 0.
void orc_pack(const uint8_t* codes, uint64_t n, uint32_t bits, uint32_t* words) {
    const uint64_t nw = orc_packed_words(n, bits);
    for (uint64_t w = 0; w < nw; ++w) words[w] = 0u;
    for (uint64_t i = 0; i < n; ++i) {
        for (uint32_t t = 0; t < bits; ++t) {
            const uint64_t pos = i * bits + t;
            const uint32_t bit = (codes[i] >> t) & 1u;
            words[pos >> 5] |= bit << (pos & 31u);
        }
    }
}

void orc_unpack(const uint32_t* words, uint64_t n, uint32_t bits, uint8_t* codes) {
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t k = 0;
        for (uint32_t t = 0; t < bits; ++t) {
            const uint64_t pos = i * bits + t;
            k |= ((words[pos >> 5] >> (pos & 31u)) & 1u) << t;
        }
        codes[i] = (uint8_t)k;
    }
}

// Worker side, whole: scales (computed, or taken from scales_in when it is
// not null), codes, packed stream.  `codes_tmp` is caller-provided scratch of
// n bytes.
void orc_quantize(const float* g, uint64_t n, uint32_t bits, uint32_t bucket, int scale_mode,
                  uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                  const float* scales_in, uint32_t* packed, float* scales_out, uint8_t* codes_tmp) {
    if (scales_in) {
        const uint64_t nb = orc_num_buckets(n, bucket);
        for (uint64_t k = 0; k < nb; ++k) scales_out[k] = scales_in[k];
    } else {
        orc_bucket_scales(g, n, bucket, scale_mode, scales_out);
    }
    orc_quantize_codes(g, n, bits, bucket, seed, iteration, worker, elem_base, scales_out, codes_tmp);
    orc_pack(codes_tmp, n, bits, packed);
}

// De-quantize one worker's stream to fp32 values.
void orc_dequantize(const uint32_t* packed, const float* scales, uint64_t n, uint32_t bits,
                    uint32_t bucket, float* out, uint8_t* codes_tmp) {
    orc_unpack(packed, n, bits, codes_tmp);
    for (uint64_t i = 0; i < n; ++i) {
        const float d = dequant_step(scales[i / bucket], bits);
        out[i] = dequant_value(codes_tmp[i], d, bits);
    }
}

// Server side: de-quantize the W workers' streams, sum them in worker order
// with one fused multiply-add per worker, and apply the SGD step with the
// mean:  p <- p - (lr/W) * sum_w v_w   (Algorithm 1: the server averages the
// de-quantized gradients; the update rule is the worker's last line).
void orc_aggregate_update(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                          uint64_t n, uint32_t bits, uint32_t bucket, float lr, float* params) {
    const int L = (int)((1u << bits) - 1u);
    const float c = lr / (float)W;
    for (uint64_t i = 0; i < n; ++i) {
        float acc = 0.0f;
        for (uint32_t w = 0; w < W; ++w) {
            uint32_t k = 0;
            for (uint32_t t = 0; t < bits; ++t) {
                const uint64_t pos = i * bits + t;
                k |= ((packed[w][pos >> 5] >> (pos & 31u)) & 1u) << t;
            }
            const float d = scales[w][i / bucket] / (float)L;
            acc = std::fmaf((float)(2 * (int)k - L), d, acc);
        }
        params[i] = std::fmaf(-c, acc, params[i]);
    }
}

// ---- the paper's full exchange: the server sends the quantized MEAN back (Algorithm 1) ----------
// ReceiveQGThenSendQG: g^m <- sum_p De-quantize(gbar_p) / P;  gbar^m <- Quantize(g^m, K);  send.
// WorkerIterate:       g^m <- De-quantize(gbar^m);  w <- w - eta g^m.
//
// Reading: the division by P is applied to the bucket RANGE, not to every element.  A range-linear
// grid is scale-equivariant: the codes of the sum on the grid over [-S, S], S = max|sum|, are the
// codes of the mean on the grid over [-S/P, S/P].  So the server quantizes the fp32 sum (ordered fma
// chain, as in orc_aggregate_update) with S, and stores S / P as the bucket scale.

void orc_aggregate_sum(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                       uint64_t n, uint32_t bits, uint32_t bucket, float* sum_out) {
    const int L = (int)((1u << bits) - 1u);
    for (uint64_t i = 0; i < n; ++i) {
        float acc = 0.0f;
        for (uint32_t w = 0; w < W; ++w) {
            uint32_t k = 0;
            for (uint32_t t = 0; t < bits; ++t) {
                const uint64_t pos = i * bits + t;
                k |= ((packed[w][pos >> 5] >> (pos & 31u)) & 1u) << t;
            }
            const float d = scales[w][i / bucket] / (float)L;
            acc = std::fmaf((float)(2 * (int)k - L), d, acc);
        }
        sum_out[i] = acc;
    }
}

// sum_tmp: n floats of scratch; codes_tmp: n bytes of scratch.
void orc_aggregate_requantize(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                              uint64_t n, uint32_t bits, uint32_t bucket,
                              uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                              uint32_t* packed_out, float* scales_out, float* sum_tmp, uint8_t* codes_tmp) {
    orc_aggregate_sum(packed, scales, W, n, bits, bucket, sum_tmp);
    orc_bucket_scales(sum_tmp, n, bucket, 0, scales_out);                       // S = max|sum| per bucket
    orc_quantize_codes(sum_tmp, n, bits, bucket, seed, iteration, worker, elem_base, scales_out, codes_tmp);
    orc_pack(codes_tmp, n, bits, packed_out);
    const uint64_t nb = orc_num_buckets(n, bucket);
    for (uint64_t k = 0; k < nb; ++k) scales_out[k] = scales_out[k] / (float)W;   // range of the mean
}

// Worker side of the exchange: w <- w - eta * De-quantize(gbar).
void orc_dequantize_update(const uint32_t* packed, const float* scales, uint64_t n, uint32_t bits,
                           uint32_t bucket, float lr, float* params) {
    const int L = (int)((1u << bits) - 1u);
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t k = 0;
        for (uint32_t t = 0; t < bits; ++t) {
            const uint64_t pos = i * bits + t;
            k |= ((packed[pos >> 5] >> (pos & 31u)) & 1u) << t;
        }
        const float d = scales[i / bucket] / (float)L;
        const float v = (float)(2 * (int)k - L) * d;
        params[i] = std::fmaf(-lr, v, params[i]);
    }
}

// The server's mean gradient itself (Algorithm 1, ReceiveQGThenSendQG: g^m <- sum_p De-quantize / P),
// for callers whose optimizer is not the paper's plain SGD step: the worker-order fma chain of
// orc_aggregate_update, divided by W with one IEEE fp32 division.  W = 1 is De-quantize.
void orc_aggregate_mean(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                        uint64_t n, uint32_t bits, uint32_t bucket, float* mean_out) {
    orc_aggregate_sum(packed, scales, W, n, bits, bucket, mean_out);
    for (uint64_t i = 0; i < n; ++i) mean_out[i] = mean_out[i] / (float)W;
}

// Layers that are sent uncompressed (the paper quantizes only its two large fully connected layers
// and communicates the other parameters "without any compression", Section 4.1): the server averages
// the raw fp32 gradients in worker order and applies the same update.
void orc_average_update_raw(const float* const* grads, uint32_t W, uint64_t n, float lr, float* params) {
    const float c = lr / (float)W;
    for (uint64_t i = 0; i < n; ++i) {
        float acc = 0.0f;
        for (uint32_t w = 0; w < W; ++w) acc = acc + grads[w][i];
        params[i] = std::fmaf(-c, acc, params[i]);
    }
}

// ---- The footnote read literally: deterministic range-linear encode over [min, max] ---------------
// Section 3.2's footnote names a range-linear Encode / Decode: the tensor's range [min, max] is cut
// into 2^K - 1 equal steps, a value is stored as the index of the nearest level and restored as
// min + index * step.  No random numbers.  Here the range is taken per bucket (bucket >= n gives the
// paper's one range per tensor); a bound that is zero is stored as +0.

// ranges[2k] = min, ranges[2k+1] = max of bucket k
void orc_minmax_ranges(const float* g, uint64_t n, uint32_t bucket, float* ranges) {
    const uint64_t nb = (n + bucket - 1) / bucket;
    for (uint64_t k = 0; k < nb; ++k) {
        const uint64_t lo_i = k * bucket;
        const uint64_t hi_i = (lo_i + bucket < n) ? lo_i + bucket : n;
        float mn = g[lo_i], mx = g[lo_i];
        for (uint64_t i = lo_i + 1; i < hi_i; ++i) {
            if (g[i] < mn) mn = g[i];
            if (g[i] > mx) mx = g[i];
        }
        if (mn == 0.0f) mn = 0.0f;   // -0 -> +0
        if (mx == 0.0f) mx = 0.0f;
        ranges[2 * k] = mn;
        ranges[2 * k + 1] = mx;
    }
}

// Index of the level nearest to x on the grid of 2^bits levels over [mn, mx]; ties go to the even
// index (the default IEEE rounding of nearbyintf).  A range narrower than 2^-96 has one level.
uint32_t orc_nearest_code(float x, float mn, float mx, uint32_t bits) {
    const float L = (float)((1u << bits) - 1u);
    const float r = mx - mn;
    const float a = (r >= 0x1p-96f) ? L / r : 0.0f;
    const float d = x - mn;
    float u = std::nearbyintf(d * a);
    if (!(u >= 0.0f)) u = 0.0f;
    if (u > L) u = L;
    return (uint32_t)u;
}

// Decode: min + index * step, step = (max - min) / (2^bits - 1), one fused multiply-add.
float orc_minmax_level_value(uint32_t k, float mn, float mx, uint32_t bits) {
    const float L = (float)((1u << bits) - 1u);
    const float step = (mx - mn) / L;
    return std::fmaf((float)k, step, mn);
}

void orc_quantize_minmax(const float* g, uint64_t n, uint32_t bits, uint32_t bucket, uint32_t* packed,
                         float* ranges, uint8_t* codes_out) {
    orc_minmax_ranges(g, n, bucket, ranges);
    uint8_t* codes = codes_out ? codes_out : new uint8_t[n ? n : 1];
    for (uint64_t i = 0; i < n; ++i) {
        const uint64_t k = i / bucket;
        codes[i] = (uint8_t)orc_nearest_code(g[i], ranges[2 * k], ranges[2 * k + 1], bits);
    }
    orc_pack(codes, n, bits, packed);
    if (!codes_out) delete[] codes;
}

void orc_dequantize_minmax(const uint32_t* packed, const float* ranges, uint64_t n, uint32_t bits,
                           uint32_t bucket, float* out) {
    uint8_t* codes = new uint8_t[n ? n : 1];
    orc_unpack(packed, n, bits, codes);
    for (uint64_t i = 0; i < n; ++i) {
        const uint64_t k = i / bucket;
        out[i] = orc_minmax_level_value(codes[i], ranges[2 * k], ranges[2 * k + 1], bits);
    }
    delete[] codes;
}

// Server step for this encoding: de-quantize every worker's gradient, add them up in worker order,
// average and update (Algorithm 1, ReceiveQGThenSendQG and the last line of WorkerIterate).
void orc_aggregate_update_minmax(const uint32_t* const* packed, const float* const* ranges, uint32_t W,
                                 uint64_t n, uint32_t bits, uint32_t bucket, float lr, float* params) {
    float* sum = new float[n ? n : 1];
    float* v = new float[n ? n : 1];
    for (uint64_t i = 0; i < n; ++i) sum[i] = 0.0f;
    for (uint32_t w = 0; w < W; ++w) {
        orc_dequantize_minmax(packed[w], ranges[w], n, bits, bucket, v);
        for (uint64_t i = 0; i < n; ++i) sum[i] = sum[i] + v[i];
    }
    const float c = lr / (float)W;
    for (uint64_t i = 0; i < n; ++i) params[i] = std::fmaf(-c, sum[i], params[i]);
    delete[] sum;
    delete[] v;
}

// The paper's full exchange with this encoding (Algorithm 1, ReceiveQGThenSendQG): the server adds the
// workers' de-quantized gradients in worker order, encodes the sum over its own per-bucket [min, max]
// and stores the range divided by W -- a range-linear grid is equivariant under positive scaling, so
// the codes of the sum over [mn, mx] are the codes of the mean over [mn / W, mx / W].
void orc_aggregate_sum_minmax(const uint32_t* const* packed, const float* const* ranges, uint32_t W,
                              uint64_t n, uint32_t bits, uint32_t bucket, float* sum) {
    float* v = new float[n ? n : 1];
    for (uint64_t i = 0; i < n; ++i) sum[i] = 0.0f;
    for (uint32_t w = 0; w < W; ++w) {
        orc_dequantize_minmax(packed[w], ranges[w], n, bits, bucket, v);
        for (uint64_t i = 0; i < n; ++i) sum[i] = sum[i] + v[i];
    }
    delete[] v;
}

void orc_aggregate_requantize_minmax(const uint32_t* const* packed, const float* const* ranges, uint32_t W,
                                     uint64_t n, uint32_t bits, uint32_t bucket, uint32_t* packed_out,
                                     float* ranges_out) {
    float* sum = new float[n ? n : 1];
    orc_aggregate_sum_minmax(packed, ranges, W, n, bits, bucket, sum);
    orc_quantize_minmax(sum, n, bits, bucket, packed_out, ranges_out, nullptr);
    const uint64_t nb = (n + bucket - 1) / bucket;
    for (uint64_t k = 0; k < 2 * nb; ++k) ranges_out[k] = ranges_out[k] / (float)W;
    delete[] sum;
}

// The same server step evaluated from its plain definition in fp64 (no
// ordering, no fp32 rounding until the end): used to pin the fp32 chain.
void orc_aggregate_update_f64(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                              uint64_t n, uint32_t bits, uint32_t bucket, double lr,
                              const float* params_in, double* params_out) {
    const double L = (double)((1u << bits) - 1u);
    for (uint64_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (uint32_t w = 0; w < W; ++w) {
            uint32_t k = 0;
            for (uint32_t t = 0; t < bits; ++t) {
                const uint64_t pos = i * bits + t;
                k |= ((packed[w][pos >> 5] >> (pos & 31u)) & 1u) << t;
            }
            acc += (double)scales[w][i / bucket] * (2.0 * (double)k - L) / L;
        }
        params_out[i] = (double)params_in[i] - lr * acc / (double)W;
    }
}

}  // extern "C"
