/*
 * psb_oracle.cpp -- see psb_oracle.h.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain loops, one step of the method per statement, in the order and the
 * notation of the paper.  Build: g++ -O2 -fno-fast-math -ffp-contract=off
 * -fopenmp (OpenMP only spreads independent output elements over cores; the
 * arithmetic of one output element is strictly sequential).
 */
#include "psb_oracle.h"

#include <cmath>
#include <cstdlib>
#include <cstring>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------------------
 * Number system: Sect. 3.1, Eq. (numbersystem) and the definitions of s, e, p.
 * ------------------------------------------------------------------------- */
extern "C" int psbo_decode(float w, int32_t* s, int32_t* e, double* p)
{
    const int cls = std::fpclassify(w);
    if (cls == FP_NAN || cls == FP_INFINITE) return PSBO_NONFINITE;
    if (cls == FP_ZERO) return PSBO_ZERO;

    const double a = std::fabs((double)w);          /* |w|, exact in binary64       */
    int ex = 0;
    (void)std::frexp(a, &ex);                       /* a = m * 2^ex, m in [0.5, 1)  */
    const int e_ = ex - 1;                          /* e = floor(log2 |w|)          */
    const double p_ = std::ldexp(a, -e_) - 1.0;     /* p = |w| / 2^e - 1  (exact)   */

    if (s) *s = (w < 0.0f) ? -1 : 1;
    if (e) *e = e_;
    if (p) *p = p_;
    return (cls == FP_SUBNORMAL) ? PSBO_SUBNORMAL : PSBO_NORMAL;
}

/* ---------------------------------------------------------------------------
 * Philox4x32-10, written from the published description: ten rounds; a round
 * multiplies words 0 and 2 by two fixed odd constants, keeps the low halves
 * and xors the high halves with the two other words and the round key; the
 * key is advanced by two Weyl constants between rounds.
 * ------------------------------------------------------------------------- */
extern "C" void psbo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t MUL_A = 0xD2511F53u;   /* multiplies word 0 */
    const uint64_t MUL_B = 0xCD9E8D57u;   /* multiplies word 2 */
    const uint32_t WEYL_0 = 0x9E3779B9u;  /* golden ratio      */
    const uint32_t WEYL_1 = 0xBB67AE85u;  /* sqrt(3) - 1       */

    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += WEYL_0; k1 += WEYL_1; }
        const uint64_t prod_a = MUL_A * (uint64_t)c0;
        const uint64_t prod_b = MUL_B * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(prod_b >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)prod_b;
        const uint32_t n2 = (uint32_t)(prod_a >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)prod_a;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

extern "C" uint32_t psbo_uniform(uint64_t seed, uint32_t layer_id, uint32_t o, uint32_t k, uint32_t s)
{
    const uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFull), (uint32_t)(seed >> 32) };
    const uint32_t ctr[4] = { o, k, s / 4u, layer_id };
    uint32_t block[4];
    psbo_philox4x32_10(ctr, key, block);
    return block[s % 4u];
}

extern "C" uint32_t psbo_uniform7(uint64_t seed, uint32_t layer_id, uint32_t o, uint32_t k, uint32_t s)
{
    const uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFull), (uint32_t)(seed >> 32) };
    const uint32_t ctr[4] = { o, k, s / 16u, layer_id };
    uint32_t block[4];
    psbo_philox4x32_10(ctr, key, block);
    const uint32_t byte_index = s % 16u;
    const uint32_t byte = (block[byte_index / 4u] >> (8u * (byte_index % 4u))) & 0xFFu;
    return byte & 0x7Fu;
}

/* ---------------------------------------------------------------------------
 * Encoding of a layer.
 *
 * Paper: weights become (s, e, p) (Sect. 3.1); exponents are stored with
 * k_e bits, 4 being enough (Sect. 4.4, suppl. "Stochastic multiplier"); the
 * width of the integers limits the exponents (caption of the multiplier
 * figure); an integer shifted too far is simply 0 (caption of Fig.
 * numbersystem).
 *
 * Reading: activations are integers, so the shift must be >= 0.  Shifts are
 * taken relative to a per-layer e_min and 2^e_min goes into the final rescale.
 * e_top = largest e of a normal non-zero weight.  e_min is the SMALLEST
 * integer in [e_top - (2^k_e - 1), e_top] for which
 *     x_absmax * s_max * max_oc  sum_{k : e_k >= e_min} 2^(e_k - e_min + 1)
 * does not exceed 2^31 - 1 (every sample taking the larger shift, every
 * activation at its largest magnitude: then no int32 accumulator can wrap).
 * Weights with e_k < e_min, and all subnormal weights, are flushed to zero.
 * Zero weights are not live either and are never sampled.
 * ------------------------------------------------------------------------- */
extern "C" int psbo_quantize(const float* w, int32_t oc, int32_t K, int32_t prob_bits, int32_t exp_bits,
                             int32_t x_absmax, int32_t s_max, psbo_weights* out)
{
    if (!w || !out || oc <= 0 || K <= 0) return PSBO_ERR_ARG;
    if (prob_bits < 1 || prob_bits > 23) return PSBO_ERR_VALUE;
    if (exp_bits <= 0) exp_bits = 4;
    if (exp_bits > 5 || x_absmax <= 0 || x_absmax > 128 || s_max <= 0 || s_max > 255) return PSBO_ERR_VALUE;

    const int64_t nw = (int64_t)oc * K;
    int32_t* e_all = (int32_t*)std::malloc(sizeof(int32_t) * nw);
    int*     cls   = (int*)std::malloc(sizeof(int) * nw);
    out->oc = oc; out->K = K; out->prob_bits = prob_bits;
    out->sign  = (int8_t*)std::calloc(nw, sizeof(int8_t));
    out->shift = (int32_t*)std::calloc(nw, sizeof(int32_t));
    out->p     = (double*)std::calloc(nw, sizeof(double));

    bool any = false;
    int32_t e_top = 0;
    for (int64_t i = 0; i < nw; ++i) {
        int32_t s = 0, e = 0; double p = 0.0;
        cls[i] = psbo_decode(w[i], &s, &e, &p);
        if (cls[i] == PSBO_NONFINITE) {
            std::free(e_all); std::free(cls); psbo_weights_free(out);
            return PSBO_ERR_VALUE;
        }
        if (prob_bits < 23 && cls[i] == PSBO_NORMAL) {
            /* Sect. 4.4: regular grid with p = 0, without p = 1 (p = 1 is the next exponent);
             * nearbyint rounds half to even in the default rounding mode */
            const double scale = std::ldexp(1.0, prob_bits);
            double P = std::nearbyint(p * scale);
            if (P >= scale) { P = 0.0; e += 1; }
            p = P / scale;
            if (e > 127) {             /* rounded past the largest binary32 exponent */
                std::free(e_all); std::free(cls); psbo_weights_free(out);
                return PSBO_ERR_VALUE;
            }
        }
        e_all[i] = e;
        out->sign[i] = (int8_t)s;      /* provisional; cleared below if not live */
        out->p[i] = p;
        if (cls[i] == PSBO_NORMAL) {
            if (!any || e > e_top) e_top = e;
            any = true;
        }
    }

    int32_t e_min = e_top;
    bool found = !any;                 /* nothing to sample: any window is safe  */
    if (any) {
        const int32_t window = (1 << exp_bits) - 1;
        for (int32_t cand = e_top - window; cand <= e_top && !found; ++cand) {
            unsigned __int128 worst = 0;
            for (int32_t o = 0; o < oc; ++o) {
                unsigned __int128 sum = 0;
                for (int32_t k = 0; k < K; ++k) {
                    const int64_t i = (int64_t)o * K + k;
                    if (cls[i] == PSBO_NORMAL && e_all[i] >= cand)
                        sum += (unsigned __int128)1 << (e_all[i] - cand + 1);
                }
                if (sum > worst) worst = sum;
            }
            const unsigned __int128 bound = worst * (unsigned)x_absmax * (unsigned)s_max;
            if (bound <= (unsigned __int128)2147483647u) { e_min = cand; found = true; }
        }
    }
    if (!found) {
        std::free(e_all); std::free(cls); psbo_weights_free(out);
        return PSBO_ERR_OVERFLOW_UNSAFE;
    }

    psbo_winfo info; info.e_top = e_top; info.e_min = e_min;
    info.n_zero = info.n_flushed = info.n_live = 0;
    for (int64_t i = 0; i < nw; ++i) {
        if (cls[i] == PSBO_ZERO) {
            info.n_zero++; out->sign[i] = 0; out->p[i] = 0.0;
        } else if (cls[i] == PSBO_SUBNORMAL || e_all[i] < e_min) {
            info.n_flushed++; out->sign[i] = 0; out->p[i] = 0.0;
        } else {
            info.n_live++; out->shift[i] = e_all[i] - e_min;
        }
    }
    out->info = info;
    std::free(e_all); std::free(cls);
    return PSBO_OK;
}

extern "C" void psbo_weights_free(psbo_weights* q)
{
    if (!q) return;
    std::free(q->sign);  q->sign = nullptr;
    std::free(q->shift); q->shift = nullptr;
    std::free(q->p);     q->p = nullptr;
}

/* ---------------------------------------------------------------------------
 * One product of the sum, samples [from, to):
 *     sum_s  sigma * ( x << (shift + B^(s)) ),   Pr(B = 1) = p
 * (Sect. 3.1: the bit shift 2^(e+1) is chosen with probability p, 2^e with
 * 1-p; one random bit per shift instruction, Sect. 2).  The random bit is
 * B = [ U < p ] with U = u / 2^32 uniform on [0,1).
 * Returned exactly (int64); negative x is handled as a multiplication by the
 * power of two, which is what a left shift means on a two's complement value.
 * ------------------------------------------------------------------------- */
static int64_t product_samples(int32_t x, int sigma, int32_t shift, double p, int32_t prob_bits,
                               int32_t from, int32_t to,
                               uint64_t seed, uint32_t layer_id, uint32_t o, uint32_t k,
                               const uint32_t* u_row /* [S] or NULL */)
{
    int64_t sum = 0;
    for (int32_t s = from; s < to; ++s) {
        double U;                                   /* uniform on [0,1) */
        if (prob_bits >= 8) {      /* p exact, or on a grid of 8..22 bits: a k_p-bit comparator on the top k_p bits of u */
            const uint32_t u = u_row ? u_row[s] : psbo_uniform(seed, layer_id, o, k, (uint32_t)s);
            U = (double)u / 4294967296.0;
        } else {
            const uint32_t u7 = u_row ? u_row[s] : psbo_uniform7(seed, layer_id, o, k, (uint32_t)s);
            U = (double)u7 / 128.0;
        }
        const int B = (U < p) ? 1 : 0;
        sum += (int64_t)sigma * (int64_t)x * ((int64_t)1 << (shift + B));
    }
    return sum;
}

extern "C" int psbo_linear(const psbo_weights* q, const int8_t* x, int32_t B, int32_t S,
                           uint64_t seed, uint32_t layer_id, const uint32_t* u_table,
                           int32_t* acc, int64_t* overflow)
{
    if (!q || !x || !acc || B <= 0 || S <= 0) return PSBO_ERR_ARG;
    const int32_t OC = q->oc, K = q->K;
    int64_t n_over = 0;
#pragma omp parallel for collapse(2) reduction(+ : n_over) schedule(static)
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t oc = 0; oc < OC; ++oc) {
            const uint32_t o = (uint32_t)((int64_t)b * OC + oc);
            int64_t exact = 0;       /* the sum as an integer                  */
            uint32_t wrapped = 0;    /* the same sum in a 32-bit register      */
            for (int32_t k = 0; k < K; ++k) {
                const int64_t wi = (int64_t)oc * K + k;
                if (q->sign[wi] == 0) continue;           /* not live: never sampled */
                const uint32_t* u_row = u_table ? u_table + ((int64_t)o * K + k) * S : nullptr;
                const int64_t t = product_samples(x[(int64_t)b * K + k], q->sign[wi], q->shift[wi],
                                                  q->p[wi], q->prob_bits, 0, S, seed, layer_id, o, (uint32_t)k, u_row);
                exact += t;
                wrapped += (uint32_t)t;
            }
            if (exact < INT32_MIN || exact > INT32_MAX) n_over++;
            acc[o] = (int32_t)wrapped;
        }
    }
    if (overflow) *overflow = n_over;
    return PSBO_OK;
}

extern "C" int psbo_conv2d(const psbo_weights* q, const psbo_wshape* ws, const int8_t* x,
                           const psbo_geom* g, int32_t S_uniform, int32_t s_max,
                           const uint8_t* budget_to, const uint8_t* budget_from,
                           uint64_t seed, uint32_t layer_id,
                           const int64_t* points, int64_t n_points,
                           int32_t* acc, int64_t* overflow, int64_t* n_smac)
{
    if (!q || !ws || !x || !g || !acc) return PSBO_ERR_ARG;
    const int32_t OC = ws->oc, C = ws->cin, KH = ws->kh, KW = ws->kw, G = ws->groups;
    if (OC <= 0 || C <= 0 || KH <= 0 || KW <= 0 || G <= 0 || C % G || OC % G) return PSBO_ERR_ARG;
    const int32_t Cg = C / G, OCg = OC / G, K = Cg * KH * KW;
    if (q->oc != OC || q->K != K) return PSBO_ERR_ARG;
    const int32_t N = g->n, H = g->h, W = g->w;
    if (N <= 0 || H <= 0 || W <= 0 || g->stride_h <= 0 || g->stride_w <= 0 || g->pad_h < 0 || g->pad_w < 0)
        return PSBO_ERR_ARG;
    if (H + 2 * g->pad_h < KH || W + 2 * g->pad_w < KW) return PSBO_ERR_ARG;
    const int32_t OH = (H + 2 * g->pad_h - KH) / g->stride_h + 1;
    const int32_t OW = (W + 2 * g->pad_w - KW) / g->stride_w + 1;
    if (!budget_to && S_uniform <= 0) return PSBO_ERR_ARG;
    if (budget_from && !budget_to) return PSBO_ERR_ARG;
    if (points && n_points < 0) return PSBO_ERR_ARG;

    const int64_t total = (int64_t)N * OC * OH * OW;
    const int64_t count = points ? n_points : total;
    int64_t n_over = 0, n_mac = 0;

#pragma omp parallel for reduction(+ : n_over, n_mac) schedule(dynamic, 64)
    for (int64_t idx = 0; idx < count; ++idx) {
        const int64_t flat = points ? points[idx] : idx;     /* ((n*OC+oc)*OH+oy)*OW+ox */
        const int32_t ox = (int32_t)(flat % OW);
        const int32_t oy = (int32_t)((flat / OW) % OH);
        const int32_t oc = (int32_t)((flat / ((int64_t)OW * OH)) % OC);
        const int32_t n  = (int32_t)(flat / ((int64_t)OW * OH * OC));
        const uint32_t o = (uint32_t)flat;

        /* sample range of this output pixel (shared by all channels) */
        const int64_t pix = ((int64_t)n * OH + oy) * OW + ox;
        int32_t to = budget_to ? budget_to[pix] : S_uniform;
        if (to > s_max) to = s_max;
        int32_t from = budget_from ? budget_from[pix] : 0;
        if (from > to) from = to;

        const int32_t grp = oc / OCg;
        int64_t exact = 0;
        uint32_t wrapped = 0;
        int64_t taps = 0;
        for (int32_t ci = 0; ci < Cg; ++ci)
            for (int32_t kh = 0; kh < KH; ++kh)
                for (int32_t kw = 0; kw < KW; ++kw) {
                    const int32_t k = (ci * KH + kh) * KW + kw;
                    const int64_t wi = (int64_t)oc * K + k;
                    if (q->sign[wi] == 0) continue;                 /* not live     */
                    const int32_t iy = oy * g->stride_h - g->pad_h + kh;
                    const int32_t ix = ox * g->stride_w - g->pad_w + kw;
                    if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;   /* padding: x = 0 */
                    const int32_t c = grp * Cg + ci;
                    const int32_t xv = x[(((int64_t)n * C + c) * H + iy) * W + ix];
                    const int64_t t = product_samples(xv, q->sign[wi], q->shift[wi], q->p[wi], q->prob_bits,
                                                      from, to, seed, layer_id, o, (uint32_t)k, nullptr);
                    exact += t;
                    wrapped += (uint32_t)t;
                    taps++;
                }
        n_mac += taps * (to - from);

        const int64_t dst = points ? idx : flat;
        if (budget_from) {                       /* refinement: add to what is there */
            exact += acc[dst];
            wrapped += (uint32_t)acc[dst];
        }
        if (exact < INT32_MIN || exact > INT32_MAX) n_over++;
        acc[dst] = (int32_t)wrapped;
    }
    if (overflow) *overflow = n_over;
    if (n_smac) *n_smac = n_mac;
    return PSBO_OK;
}

/* ---------------------------------------------------------------------------
 * Shared-filter mode: Eq. (numbersystem:simulation),
 *     w  ->  s * 2^e * ( B_{n,p} / n + 1 ),
 * one binomial count per WEIGHT and per pass, after which the layer is an
 * ordinary convolution with the sampled filter (Sect. 4.1 "Setup": the filter is
 * sampled directly; suppl. "Efficient simulation of the forward pass", Eq.
 * (binomial)).  In integers, in units of 2^e_min and before the division by n:
 *     W[oc][k] = sigma * 2^shift * ( n + B ),   B = #{ i in [from,to) : U_i < p },
 * n = to - from.  B is the sum of the same kind of Bernoulli draws the
 * per-product mode uses, taken from the stream of "output element" oc:
 * U_i = uniform(seed, layer_id, o := oc, k, i).  All output pixels of a channel
 * therefore see the same filter, which is what the simulation does and what the
 * per-product mode does not.
 * ------------------------------------------------------------------------- */
static int32_t filter_count(const psbo_weights* q, int64_t wi, uint32_t oc, uint32_t k, int32_t from, int32_t to,
                            uint64_t seed, uint32_t layer_id, const uint32_t* u_row)
{
    int32_t B = 0;
    for (int32_t s = from; s < to; ++s) {
        double U;
        if (q->prob_bits >= 8) {
            const uint32_t u = u_row ? u_row[s] : psbo_uniform(seed, layer_id, oc, k, (uint32_t)s);
            U = (double)u / 4294967296.0;
        } else {
            const uint32_t u7 = u_row ? u_row[s] : psbo_uniform7(seed, layer_id, oc, k, (uint32_t)s);
            U = (double)u7 / 128.0;
        }
        if (U < q->p[wi]) B++;
    }
    return B;
}

extern "C" int psbo_sample_filter(const psbo_weights* q, int32_t from, int32_t to, uint64_t seed,
                                  uint32_t layer_id, const uint32_t* u_table, int32_t table_S, int64_t* W)
{
    if (!q || !W || from < 0 || to < from) return PSBO_ERR_ARG;
    if (u_table && to > table_S) return PSBO_ERR_ARG;
    for (int32_t oc = 0; oc < q->oc; ++oc)
        for (int32_t k = 0; k < q->K; ++k) {
            const int64_t wi = (int64_t)oc * q->K + k;
            if (q->sign[wi] == 0) { W[wi] = 0; continue; }
            const uint32_t* u_row = u_table ? u_table + wi * table_S : nullptr;
            const int32_t B = filter_count(q, wi, (uint32_t)oc, (uint32_t)k, from, to, seed, layer_id, u_row);
            W[wi] = (int64_t)q->sign[wi] * ((int64_t)1 << q->shift[wi]) * (int64_t)((to - from) + B);
        }
    return PSBO_OK;
}

extern "C" int psbo_conv2d_shared(const psbo_weights* q, const psbo_wshape* ws, const int8_t* x,
                                  const psbo_geom* g, int32_t S_uniform, int32_t s_max,
                                  const uint8_t* budget_to, const uint8_t* budget_from,
                                  uint64_t seed, uint32_t layer_id, const int64_t* points, int64_t n_points,
                                  int32_t* acc, int64_t* overflow)
{
    if (!q || !ws || !x || !g || !acc) return PSBO_ERR_ARG;
    const int32_t OC = ws->oc, C = ws->cin, KH = ws->kh, KW = ws->kw, G = ws->groups;
    if (OC <= 0 || C <= 0 || KH <= 0 || KW <= 0 || G <= 0 || C % G || OC % G) return PSBO_ERR_ARG;
    const int32_t Cg = C / G, OCg = OC / G, K = Cg * KH * KW;
    if (q->oc != OC || q->K != K) return PSBO_ERR_ARG;
    const int32_t N = g->n, H = g->h, Wd = g->w;
    if (N <= 0 || H <= 0 || Wd <= 0 || g->stride_h <= 0 || g->stride_w <= 0 || g->pad_h < 0 || g->pad_w < 0)
        return PSBO_ERR_ARG;
    if (H + 2 * g->pad_h < KH || Wd + 2 * g->pad_w < KW) return PSBO_ERR_ARG;
    const int32_t OH = (H + 2 * g->pad_h - KH) / g->stride_h + 1;
    const int32_t OW = (Wd + 2 * g->pad_w - KW) / g->stride_w + 1;
    if (!budget_to && S_uniform <= 0) return PSBO_ERR_ARG;
    if (budget_from && !budget_to) return PSBO_ERR_ARG;
    if (s_max <= 0 || s_max > 255) return PSBO_ERR_ARG;
    if (points && n_points < 0) return PSBO_ERR_ARG;

    /* prefix counts: cnt[wi][s] = number of ones among samples 0 .. s-1 of weight wi */
    const int64_t nw = (int64_t)OC * K;
    const int32_t smax_used = budget_to ? s_max : (S_uniform < s_max ? S_uniform : s_max);
    const int64_t row = (int64_t)smax_used + 1;
    int16_t* cnt = (int16_t*)std::calloc((size_t)(nw * row), sizeof(int16_t));
    if (!cnt) return PSBO_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t wi = 0; wi < nw; ++wi) {
        if (q->sign[wi] == 0) continue;
        const uint32_t oc = (uint32_t)(wi / K), k = (uint32_t)(wi % K);
        for (int32_t s = 0; s < smax_used; ++s)
            cnt[wi * row + s + 1] = (int16_t)(cnt[wi * row + s] +
                                              filter_count(q, wi, oc, k, s, s + 1, seed, layer_id, nullptr));
    }

    const int64_t total = (int64_t)N * OC * OH * OW;
    const int64_t count = points ? n_points : total;
    int64_t n_over = 0;
#pragma omp parallel for reduction(+ : n_over) schedule(dynamic, 64)
    for (int64_t idx = 0; idx < count; ++idx) {
        const int64_t flat = points ? points[idx] : idx;
        const int64_t dst = points ? idx : flat;
        const int32_t ox = (int32_t)(flat % OW);
        const int32_t oy = (int32_t)((flat / OW) % OH);
        const int32_t oc = (int32_t)((flat / ((int64_t)OW * OH)) % OC);
        const int32_t n  = (int32_t)(flat / ((int64_t)OW * OH * OC));
        const int64_t pix = ((int64_t)n * OH + oy) * OW + ox;
        int32_t to = budget_to ? budget_to[pix] : S_uniform;
        if (to > s_max) to = s_max;
        int32_t from = budget_from ? budget_from[pix] : 0;
        if (from > to) from = to;

        const int32_t grp = oc / OCg;
        int64_t exact = 0;
        uint32_t wrapped = 0;
        for (int32_t ci = 0; ci < Cg; ++ci)
            for (int32_t kh = 0; kh < KH; ++kh)
                for (int32_t kw = 0; kw < KW; ++kw) {
                    const int32_t k = (ci * KH + kh) * KW + kw;
                    const int64_t wi = (int64_t)oc * K + k;
                    if (q->sign[wi] == 0) continue;
                    const int32_t iy = oy * g->stride_h - g->pad_h + kh;
                    const int32_t ix = ox * g->stride_w - g->pad_w + kw;
                    if (iy < 0 || iy >= H || ix < 0 || ix >= Wd) continue;
                    const int32_t c = grp * Cg + ci;
                    const int64_t xv = x[(((int64_t)n * C + c) * H + iy) * Wd + ix];
                    /* the filter value of this pixel's sample range */
                    const int64_t B = cnt[wi * row + to] - cnt[wi * row + from];
                    const int64_t Wv = (int64_t)q->sign[wi] * ((int64_t)1 << q->shift[wi]) * ((int64_t)(to - from) + B);
                    exact += xv * Wv;
                    wrapped += (uint32_t)(xv * Wv);
                }
        if (budget_from) {
            exact += acc[dst];
            wrapped += (uint32_t)acc[dst];
        }
        if (exact < INT32_MIN || exact > INT32_MAX) n_over++;
        acc[dst] = (int32_t)wrapped;
    }
    std::free(cnt);
    if (overflow) *overflow = n_over;
    return PSBO_OK;
}

/* ---------------------------------------------------------------------------
 * Normalisation by the number of samples (the ">> n" of the shift form in
 * Sect. 3.1, generalised to any sample count by a division in binary32) and
 * the per-channel affine map that stands for folded batch normalisation
 * (Sect. 3, Eq. 2).
 * ------------------------------------------------------------------------- */
extern "C" int psbo_rescale(const int32_t* acc, int32_t n, int32_t oc, int32_t spatial,
                            int32_t S_uniform, int32_t s_max, const uint8_t* budget_to,
                            int32_t e_min, const float* mult, const float* bias, float* y)
{
    if (!acc || !y || n <= 0 || oc <= 0 || spatial <= 0) return PSBO_ERR_ARG;
    if (!budget_to && S_uniform <= 0) return PSBO_ERR_ARG;
    const float default_mult = std::ldexp(1.0f, e_min);
    for (int32_t b = 0; b < n; ++b)
        for (int32_t c = 0; c < oc; ++c)
            for (int32_t sp = 0; sp < spatial; ++sp) {
                int32_t to = budget_to ? budget_to[(int64_t)b * spatial + sp] : S_uniform;
                if (to > s_max) to = s_max;
                const float inv_S = (to > 0) ? (1.0f / (float)to) : 0.0f;
                const int64_t i = ((int64_t)b * oc + c) * spatial + sp;
                volatile float a = (float)acc[i];              /* round 1: int -> binary32 */
                volatile float m = a * (mult ? mult[c] : default_mult);   /* round 2       */
                volatile float r = m * inv_S;                  /* round 3                  */
                if (bias) { volatile float t = r + bias[c]; r = t; }      /* round 4       */
                y[i] = r;
            }
    return PSBO_OK;
}

/* ---------------------------------------------------------------------------
 * Glue between layers of a network (suppl. "ReLU, Batch-Norm, and Pooling":
 * ReLU is a gate on the sign, max-pooling needs comparators, the factor of an
 * average pooling is a fixed multiplication; suppl. "Activations and
 * Accumulation": activations are stored as fixed-point integers).  Every
 * floating-point step is one binary32 operation rounded to nearest even, in
 * the order written, so that both implementations produce the same integers.
 * ------------------------------------------------------------------------- */

/* x_out = clamp( rint( g( y [+ r] ) * inv_step ), lo, hi ),  g = max(., 0) if relu else identity,
 * r = res_f32[i] or (float)res_i8[i] * res_step (one rounded multiplication), added in binary32. */
extern "C" int psbo_requantize(const float* y, const float* res_f32, const int8_t* res_i8, float res_step,
                               int relu, float inv_step, int32_t lo, int32_t hi, int64_t n, int8_t* x_out)
{
    if (!y || !x_out || n < 0 || lo < -128 || hi > 127 || lo > hi) return PSBO_ERR_ARG;
    if (res_f32 && res_i8) return PSBO_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        volatile float t = y[i];
        if (res_f32) { volatile float u = t + res_f32[i]; t = u; }
        if (res_i8) {
            volatile float r = (float)res_i8[i] * res_step;
            volatile float u = t + r;
            t = u;
        }
        if (relu && !(t > 0.0f)) t = 0.0f;             /* also maps NaN to 0 */
        volatile float scaled = t * inv_step;
        float q = std::nearbyintf(scaled);             /* ties to even in the default rounding mode */
        if (!(q >= (float)lo)) q = (float)lo;          /* NaN goes to lo */
        if (q > (float)hi) q = (float)hi;
        x_out[i] = (int8_t)(int32_t)q;
    }
    return PSBO_OK;
}

/* Max-pooling on int8, NCHW; positions in the padding do not take part. */
extern "C" int psbo_maxpool_i8(const int8_t* x, int32_t n, int32_t c, int32_t h, int32_t w, int32_t kh, int32_t kw,
                               int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int8_t* out)
{
    if (!x || !out || n <= 0 || c <= 0 || h <= 0 || w <= 0 || kh <= 0 || kw <= 0 || stride_h <= 0 || stride_w <= 0 ||
        pad_h < 0 || pad_w < 0 || 2 * pad_h > kh || 2 * pad_w > kw || h + 2 * pad_h < kh || w + 2 * pad_w < kw)
        return PSBO_ERR_ARG;
    const int32_t oh = (h + 2 * pad_h - kh) / stride_h + 1, ow = (w + 2 * pad_w - kw) / stride_w + 1;
    for (int64_t img = 0; img < (int64_t)n * c; ++img)
        for (int32_t oy = 0; oy < oh; ++oy)
            for (int32_t ox = 0; ox < ow; ++ox) {
                int32_t best = -129;
                for (int32_t dy = 0; dy < kh; ++dy)
                    for (int32_t dx = 0; dx < kw; ++dx) {
                        const int32_t iy = oy * stride_h - pad_h + dy, ix = ox * stride_w - pad_w + dx;
                        if (iy < 0 || iy >= h || ix < 0 || ix >= w) continue;
                        const int32_t v = x[(img * h + iy) * w + ix];
                        if (v > best) best = v;
                    }
                out[(img * oh + oy) * ow + ox] = (int8_t)best;   /* pad <= kernel/2: at least one position is inside */
            }
    return PSBO_OK;
}

/* Global average pooling on int8 with requantisation:
 * out[n][c] = clamp( rint( ((float)sum * fl(1/(h*w))) * scale ), lo, hi ), sum exact in int32. */
extern "C" int psbo_avgpool_requantize(const int8_t* x, int32_t n, int32_t c, int32_t h, int32_t w, float scale,
                                       int32_t lo, int32_t hi, int8_t* out)
{
    if (!x || !out || n <= 0 || c <= 0 || h <= 0 || w <= 0 || (int64_t)h * w > (1 << 23) || lo < -128 || hi > 127 ||
        lo > hi)
        return PSBO_ERR_ARG;
    const float inv_count = 1.0f / (float)(h * w);
    for (int64_t img = 0; img < (int64_t)n * c; ++img) {
        int32_t sum = 0;
        for (int64_t i = 0; i < (int64_t)h * w; ++i) sum += x[img * h * w + i];
        volatile float mean = (float)sum * inv_count;
        volatile float scaled = mean * scale;
        float q = std::nearbyintf(scaled);
        if (!(q >= (float)lo)) q = (float)lo;
        if (q > (float)hi) q = (float)hi;
        out[img] = (int8_t)(int32_t)q;
    }
    return PSBO_OK;
}

/* Budget map at another resolution (Sect. 4.5: the two kinds of regions are applied to the
 * activations of every layer): nearest source pixel, out[n][y][x] = in[n][floor(y*h/oh)][floor(x*w/ow)]. */
extern "C" int psbo_budget_resample(const uint8_t* in, int32_t n, int32_t h, int32_t w, int32_t oh, int32_t ow,
                                    uint8_t* out)
{
    if (!in || !out || n <= 0 || h <= 0 || w <= 0 || oh <= 0 || ow <= 0) return PSBO_ERR_ARG;
    for (int32_t b = 0; b < n; ++b)
        for (int32_t y = 0; y < oh; ++y)
            for (int32_t x = 0; x < ow; ++x) {
                const int64_t sy = (int64_t)y * h / oh, sx = (int64_t)x * w / ow;
                out[((int64_t)b * oh + y) * ow + x] = in[((int64_t)b * h + sy) * w + sx];
            }
    return PSBO_OK;
}

/* ---------------------------------------------------------------------------
 * Attention mask (Sect. 4.5): the pixelwise entropy of the softmax over the
 * channels of the last convolutional layer,
 *     h_xy = sum_c - softmax(a_xyc) * log(softmax(a_xyc)),
 * thresholded at the mean entropy of the image: pixels above the mean are the
 * regions that get the larger sample count.  a = (double)act * step.
 * Sect. 4.5 fixes no precision.  Reading: the entropy map and its mean are
 * binary32 tensors, like every tensor of the paper's experiments (Sect. 4.1
 * "Setup": float32), so the threshold compares binary32 values; each of them is
 * one rounding of a binary64 evaluation.
 * ------------------------------------------------------------------------- */
extern "C" int psbo_attention_budget(const int8_t* act, float step, int32_t n, int32_t c, int32_t h, int32_t w,
                                     uint8_t budget_lo, uint8_t budget_hi, float* entropy, float* mean,
                                     uint8_t* budget)
{
    if (!act || !entropy || !budget || n <= 0 || c <= 0 || h <= 0 || w <= 0) return PSBO_ERR_ARG;
    const int64_t hw = (int64_t)h * w;
    for (int32_t b = 0; b < n; ++b) {
        double total = 0.0;
        for (int64_t px = 0; px < hw; ++px) {
            double zmax = -1e300;
            for (int32_t ch = 0; ch < c; ++ch) {
                const double z = (double)act[((int64_t)b * c + ch) * hw + px] * (double)step;
                if (z > zmax) zmax = z;
            }
            double Z = 0.0;
            for (int32_t ch = 0; ch < c; ++ch)
                Z += std::exp((double)act[((int64_t)b * c + ch) * hw + px] * (double)step - zmax);
            double ent = 0.0;
            for (int32_t ch = 0; ch < c; ++ch) {
                const double z = (double)act[((int64_t)b * c + ch) * hw + px] * (double)step - zmax;
                const double p = std::exp(z) / Z;
                if (p > 0.0) ent -= p * std::log(p);
            }
            entropy[b * hw + px] = (float)ent;
            total += (double)(float)ent;
        }
        const float m = (float)(total / (double)hw);
        if (mean) mean[b] = m;
        for (int64_t px = 0; px < hw; ++px) budget[b * hw + px] = entropy[b * hw + px] > m ? budget_hi : budget_lo;
    }
    return PSBO_OK;
}

extern "C" int psbo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
