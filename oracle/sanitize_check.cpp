/*
 * sanitize_check.cpp -- TEST INFRASTRUCTURE ONLY.  Calls every function of the CPU oracle on small inputs with
 * exactly sized heap buffers, so that a build with -fsanitize=address,undefined (python oracle/build_oracle.py
 * --sanitize) reports any access outside a buffer, signed overflow, invalid shift or misaligned access in the
 * oracle.  Results are only checked for consistency between entry points (plain call = constant budget map =
 * points variant; refinement = single call); the values themselves are pinned by the Python tests.
 * Exit status 0 = nothing reported.
 */
#include "psb_oracle.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd()
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}
static float rnd_weight()
{
    const float m = 1.0f + (float)(rnd() & 0xFFFF) / 65536.0f;
    const int e = -(int)(rnd() % 9);
    const float v = std::ldexp(m, e) * ((rnd() & 1) ? -0.25f : 0.25f);
    return (rnd() % 7 == 0) ? 0.0f : v;
}
#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) { std::fprintf(stderr, "sanitize_check: %s failed (line %d)\n", #cond, __LINE__); return 1; } \
    } while (0)

static int layer_case(int N, int C, int H, int W, int OC, int KH, int KW, int G, int sh, int sw, int ph, int pw,
                      int prob_bits)
{
    const int Cg = C / G, K = Cg * KH * KW;
    const int OH = (H + 2 * ph - KH) / sh + 1, OW = (W + 2 * pw - KW) / sw + 1;
    std::vector<float> w((size_t)OC * K);
    for (auto& v : w) v = rnd_weight();
    w[0] = 1e-41f;                                        /* a subnormal: flushed */
    std::vector<int8_t> x((size_t)N * C * H * W);
    for (auto& v : x) v = (rnd() & 1) ? 0 : (int8_t)(rnd() % 255 - 127);
    const int s_max = 16;
    psbo_weights q;
    CHECK(psbo_quantize(w.data(), OC, K, prob_bits, 0, 128, s_max, &q) == PSBO_OK);
    CHECK(q.info.n_zero + q.info.n_flushed + q.info.n_live == (int64_t)OC * K);
    const psbo_wshape ws = {OC, C, KH, KW, G};
    const psbo_geom g = {N, H, W, sh, sw, ph, pw};
    const size_t total = (size_t)N * OC * OH * OW, npix = (size_t)N * OH * OW;
    std::vector<int32_t> a(total), b(total), c(total);
    int64_t over = 0, smac = 0, smac2 = 0;
    CHECK(psbo_conv2d(&q, &ws, x.data(), &g, 12, s_max, nullptr, nullptr, 77, 3, nullptr, 0, a.data(), &over, &smac) == PSBO_OK);
    CHECK(over == 0);
    std::vector<uint8_t> full(npix, 12), to(npix), from(npix);
    CHECK(psbo_conv2d(&q, &ws, x.data(), &g, 0, s_max, full.data(), nullptr, 77, 3, nullptr, 0, b.data(), &over, &smac2) == PSBO_OK);
    CHECK(std::memcmp(a.data(), b.data(), total * sizeof(int32_t)) == 0 && smac == smac2);
    for (size_t i = 0; i < npix; ++i) { to[i] = (uint8_t)(rnd() % 40); from[i] = (uint8_t)(rnd() % 9); }
    /* refinement in two calls = one call */
    CHECK(psbo_conv2d(&q, &ws, x.data(), &g, 0, s_max, to.data(), nullptr, 77, 3, nullptr, 0, a.data(), &over, nullptr) == PSBO_OK);
    CHECK(psbo_conv2d(&q, &ws, x.data(), &g, 0, s_max, from.data(), nullptr, 77, 3, nullptr, 0, b.data(), &over, nullptr) == PSBO_OK);
    /* from' = min(from, to'): pixels whose first pass went further than `to` keep what they have */
    std::vector<uint8_t> first(npix);
    for (size_t i = 0; i < npix; ++i) first[i] = (uint8_t)((from[i] < to[i] ? from[i] : to[i]) > s_max ? s_max : (from[i] < to[i] ? from[i] : to[i]));
    CHECK(psbo_conv2d(&q, &ws, x.data(), &g, 0, s_max, first.data(), nullptr, 77, 3, nullptr, 0, b.data(), &over, nullptr) == PSBO_OK);
    CHECK(psbo_conv2d(&q, &ws, x.data(), &g, 0, s_max, to.data(), first.data(), 77, 3, nullptr, 0, b.data(), &over, nullptr) == PSBO_OK);
    CHECK(std::memcmp(a.data(), b.data(), total * sizeof(int32_t)) == 0);
    /* the points variant, first and last output included */
    std::vector<int64_t> pts = {0, (int64_t)total - 1};
    for (int i = 0; i < 30; ++i) pts.push_back((int64_t)(rnd() % total));
    std::vector<int32_t> pa(pts.size());
    CHECK(psbo_conv2d(&q, &ws, x.data(), &g, 0, s_max, to.data(), nullptr, 77, 3, pts.data(), (int64_t)pts.size(), pa.data(), &over, nullptr) == PSBO_OK);
    for (size_t i = 0; i < pts.size(); ++i) CHECK(pa[i] == a[pts[i]]);
    /* shared-filter mode: the same three consistency checks */
    CHECK(psbo_conv2d_shared(&q, &ws, x.data(), &g, 0, s_max, to.data(), nullptr, 78, 4, nullptr, 0, a.data(), &over) == PSBO_OK);
    CHECK(over == 0);
    CHECK(psbo_conv2d_shared(&q, &ws, x.data(), &g, 0, s_max, first.data(), nullptr, 78, 4, nullptr, 0, c.data(), &over) == PSBO_OK);
    CHECK(psbo_conv2d_shared(&q, &ws, x.data(), &g, 0, s_max, to.data(), first.data(), 78, 4, nullptr, 0, c.data(), &over) == PSBO_OK);
    CHECK(std::memcmp(a.data(), c.data(), total * sizeof(int32_t)) == 0);
    CHECK(psbo_conv2d_shared(&q, &ws, x.data(), &g, 0, s_max, to.data(), nullptr, 78, 4, pts.data(), (int64_t)pts.size(), pa.data(), &over) == PSBO_OK);
    for (size_t i = 0; i < pts.size(); ++i) CHECK(pa[i] == a[pts[i]]);
    std::vector<int64_t> Wf((size_t)OC * K);
    CHECK(psbo_sample_filter(&q, 3, 11, 78, 4, nullptr, 0, Wf.data()) == PSBO_OK);
    /* epilogue and glue on the result */
    std::vector<float> mult(OC), bias(OC), y(total);
    for (int i = 0; i < OC; ++i) { mult[i] = 1e-3f * (float)(1 + rnd() % 9); bias[i] = (float)(rnd() % 100) * 0.01f - 0.5f; }
    CHECK(psbo_rescale(a.data(), N, OC, OH * OW, 0, s_max, to.data(), q.info.e_min, mult.data(), bias.data(), y.data()) == PSBO_OK);
    CHECK(psbo_rescale(a.data(), N, OC, OH * OW, 12, s_max, nullptr, q.info.e_min, nullptr, nullptr, y.data()) == PSBO_OK);
    std::vector<int8_t> xo(total), res(total);
    std::vector<float> resf(total);
    for (size_t i = 0; i < total; ++i) { res[i] = (int8_t)(rnd() % 255 - 127); resf[i] = (float)res[i] * 0.1f; }
    CHECK(psbo_requantize(y.data(), nullptr, res.data(), 0.05f, 1, 30.0f, 0, 127, (int64_t)total, xo.data()) == PSBO_OK);
    CHECK(psbo_requantize(y.data(), resf.data(), nullptr, 0.0f, 0, 30.0f, -128, 127, (int64_t)total, xo.data()) == PSBO_OK);
    if (OH >= 2 && OW >= 2) {
        const int ph2 = (OH + 2 - 3) / 2 + 1, pw2 = (OW + 2 - 3) / 2 + 1;
        if (OH + 2 >= 3 && OW + 2 >= 3) {
            std::vector<int8_t> pooled((size_t)N * OC * ph2 * pw2);
            CHECK(psbo_maxpool_i8(xo.data(), N, OC, OH, OW, 3, 3, 2, 2, 1, 1, pooled.data()) == PSBO_OK);
        }
    }
    std::vector<int8_t> avg((size_t)N * OC);
    CHECK(psbo_avgpool_requantize(xo.data(), N, OC, OH, OW, 1.0f, -128, 127, avg.data()) == PSBO_OK);
    std::vector<uint8_t> bud2((size_t)N * (2 * OH + 1) * (OW + 3));
    CHECK(psbo_budget_resample(to.data(), N, OH, OW, 2 * OH + 1, OW + 3, bud2.data()) == PSBO_OK);
    std::vector<float> ent(npix), mean(N);
    std::vector<uint8_t> mask(npix);
    CHECK(psbo_attention_budget(xo.data(), 0.05f, N, OC, OH, OW, 8, 16, ent.data(), mean.data(), mask.data()) == PSBO_OK);
    psbo_weights_free(&q);
    return 0;
}

int main()
{
    /* number system and generator */
    int32_t s, e; double p;
    CHECK(psbo_decode(3.0f, &s, &e, &p) == PSBO_NORMAL && s == 1 && e == 1 && p == 0.5);
    CHECK(psbo_decode(-0.0f, &s, &e, &p) == PSBO_ZERO);
    CHECK(psbo_decode(1e-42f, &s, &e, &p) == PSBO_SUBNORMAL);
    CHECK(psbo_decode(3.4e38f, &s, &e, &p) == PSBO_NORMAL && e == 127);
    const uint32_t ctr[4] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0x3FFFFFFFu, 0xFFFFFFFFu}, key[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
    uint32_t out[4];
    psbo_philox4x32_10(ctr, key, out);
    CHECK(psbo_uniform(~0ull, ~0u, ~0u, ~0u, ~0u) == out[3]);        /* s = 2^32 - 1: block 2^30 - 1, word 3 */
    CHECK(psbo_uniform7(~0ull, ~0u, ~0u, ~0u, 255u) < 128u);
    /* encoding errors and extremes */
    psbo_weights q;
    float big[4] = {3.4e38f, -3.4e38f, 1.0f, 0.0f};
    CHECK(psbo_quantize(big, 1, 4, 4, 5, 1, 1, &q) == PSBO_ERR_VALUE);            /* rounds past the largest exponent */
    CHECK(psbo_quantize(big, 1, 4, 23, 5, 1, 1, &q) == PSBO_OK);
    psbo_weights_free(&q);
    float nan4[4] = {1.0f, std::strtof("nan", nullptr), 1.0f, 1.0f};
    CHECK(psbo_quantize(nan4, 2, 2, 23, 0, 127, 8, &q) == PSBO_ERR_VALUE);
    std::vector<float> ones(1 << 16, 1.0f);
    CHECK(psbo_quantize(ones.data(), 1, 1 << 16, 23, 0, 128, 255, &q) == PSBO_ERR_OVERFLOW_UNSAFE);
    /* a linear layer with an injected uniform table */
    {
        const int B = 3, K = 5, OC = 4, S = 6;
        std::vector<float> w((size_t)OC * K);
        for (auto& v : w) v = rnd_weight();
        std::vector<int8_t> x((size_t)B * K);
        for (auto& v : x) v = (int8_t)(rnd() % 255 - 127);
        CHECK(psbo_quantize(w.data(), OC, K, 23, 0, 128, S, &q) == PSBO_OK);
        std::vector<uint32_t> table((size_t)B * OC * K * S);
        for (auto& v : table) v = rnd();
        std::vector<int32_t> acc((size_t)B * OC);
        int64_t over = 0;
        CHECK(psbo_linear(&q, x.data(), B, S, 5, 6, table.data(), acc.data(), &over) == PSBO_OK);
        CHECK(psbo_linear(&q, x.data(), B, S, 5, 6, nullptr, acc.data(), &over) == PSBO_OK);
        std::vector<int64_t> Wf((size_t)OC * K);
        std::vector<uint32_t> t2((size_t)OC * K * S);
        for (auto& v : t2) v = rnd();
        CHECK(psbo_sample_filter(&q, 0, S, 5, 6, t2.data(), S, Wf.data()) == PSBO_OK);
        psbo_weights_free(&q);
    }
    /* layers: strided, padded, grouped, rectangular, depthwise, 1x1, both uniform widths */
    if (layer_case(2, 8, 7, 9, 6, 3, 2, 2, 2, 1, 1, 1, 23)) return 1;
    if (layer_case(1, 6, 6, 5, 6, 3, 3, 6, 1, 1, 1, 1, 4)) return 1;
    if (layer_case(2, 5, 4, 4, 7, 1, 1, 1, 2, 2, 0, 0, 23)) return 1;
    if (layer_case(1, 3, 9, 8, 4, 7, 7, 1, 2, 2, 3, 3, 7)) return 1;
    if (layer_case(1, 4, 2, 3, 5, 3, 3, 1, 1, 1, 3, 3, 1)) return 1;
    std::printf("sanitize_check: ok (%d threads)\n", psbo_num_threads());
    return 0;
}
