// Drives every entry point of the oracle over ragged sizes under AddressSanitizer and
// UndefinedBehaviorSanitizer (host only).  Buffers are allocated at their exact documented sizes, so
// an access one element past an end is reported.  Prints "ok" and returns 0 when nothing was flagged.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../oracle/mqgrad_oracle.cpp"

static uint32_t lcg(uint32_t& s) { s = s * 1664525u + 1013904223u; return s; }

int main() {
    uint32_t seed = 12345u;
    const uint64_t sizes[] = {1, 2, 5, 31, 32, 33, 95, 96, 97, 1000, 4097};
    const uint32_t buckets[] = {32, 96, 512, 16384};
    for (uint64_t n : sizes) for (uint32_t bucket : buckets) for (uint32_t bits = 1; bits <= 8; ++bits) {
        const uint32_t W = 1 + bits % 3;
        const uint64_t nb = orc_num_buckets(n, bucket), nw = orc_packed_words(n, bits);
        std::vector<std::vector<float>> g(W, std::vector<float>(n));
        for (auto& v : g) for (auto& x : v) x = ((int)(lcg(seed) >> 8) - (1 << 23)) * 1e-9f;
        std::vector<std::vector<uint32_t>> pk(W, std::vector<uint32_t>(nw)), pm(W, std::vector<uint32_t>(nw));
        std::vector<std::vector<float>> sc(W, std::vector<float>(nb)), rg(W, std::vector<float>(2 * nb));
        std::vector<uint8_t> codes(n), codes2(n);
        std::vector<const uint32_t*> pkp(W), pmp(W);
        std::vector<const float*> scp(W), rgp(W), gp(W);
        for (uint32_t w = 0; w < W; ++w) {
            orc_quantize(g[w].data(), n, bits, bucket, (int)(w & 1), 99, 3, w, 8 * (n % 5), nullptr, pk[w].data(),
                         sc[w].data(), codes.data());
            orc_unpack(pk[w].data(), n, bits, codes2.data());
            for (uint64_t i = 0; i < n; ++i) if (codes[i] != codes2[i]) { std::printf("unpack mismatch\n"); return 1; }
            orc_quantize_minmax(g[w].data(), n, bits, bucket, pm[w].data(), rg[w].data(), nullptr);
            pkp[w] = pk[w].data(); scp[w] = sc[w].data(); pmp[w] = pm[w].data(); rgp[w] = rg[w].data(); gp[w] = g[w].data();
        }
        std::vector<float> params(n, 0.25f), out(n), sum(n), sc2(nb), rg2(2 * nb);
        std::vector<double> pd(n);
        std::vector<uint32_t> pk2(nw);
        orc_dequantize(pk[0].data(), sc[0].data(), n, bits, bucket, out.data(), codes.data());
        orc_aggregate_update(pkp.data(), scp.data(), W, n, bits, bucket, 0.1f, params.data());
        orc_aggregate_update_f64(pkp.data(), scp.data(), W, n, bits, bucket, 0.1, params.data(), pd.data());
        orc_aggregate_sum(pkp.data(), scp.data(), W, n, bits, bucket, sum.data());
        orc_aggregate_requantize(pkp.data(), scp.data(), W, n, bits, bucket, 7, 1, W, 0, pk2.data(), sc2.data(),
                                 sum.data(), codes.data());
        orc_dequantize_update(pk2.data(), sc2.data(), n, bits, bucket, 0.1f, params.data());
        orc_average_update_raw(gp.data(), W, n, 0.1f, params.data());
        orc_dequantize_minmax(pm[0].data(), rg[0].data(), n, bits, bucket, out.data());
        orc_aggregate_update_minmax(pmp.data(), rgp.data(), W, n, bits, bucket, 0.1f, params.data());
        orc_aggregate_sum_minmax(pmp.data(), rgp.data(), W, n, bits, bucket, sum.data());
        orc_aggregate_requantize_minmax(pmp.data(), rgp.data(), W, n, bits, bucket, pk2.data(), rg2.data());
    }
    std::printf("ok\n");
    return 0;
}
