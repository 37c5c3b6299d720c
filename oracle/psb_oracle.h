/*
 * psb_oracle.h -- CPU oracle for the stochastically binarized scalar-product
 * layer of Progressive Stochastic Binarization (Hartmann & Wand).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, sequential-by-definition
 * implementation whose only purpose is to define, for every (inputs, seed),
 * the single bit pattern the GPU library has to reproduce.  It shares no code
 * with the HIP path; nothing in the product imports, links or calls it.
 *
 * Every function names the passage of the paper it follows.  Where the paper
 * is silent the reading is stated next to the code (and listed in the design
 * document of the repository).
 *
 * Parity status: every function below is pinned by CPU tests (closed forms,
 * published known-answer vectors, brute-force enumeration, statistical bounds,
 * reduction to a textbook integer convolution).  No function is
 * "parity unpinned".
 */
#ifndef PSB_ORACLE_H
#define PSB_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* weight classes */
enum { PSBO_ZERO = 0, PSBO_NORMAL = 1, PSBO_SUBNORMAL = 2, PSBO_NONFINITE = 3 };

/* status codes (oracle-local; the GPU library has its own) */
enum { PSBO_OK = 0, PSBO_ERR_ARG = -1, PSBO_ERR_VALUE = -3, PSBO_ERR_OVERFLOW_UNSAFE = -4 };

typedef struct {
    int32_t e_top;      /* largest exponent e over normal non-zero weights      */
    int32_t e_min;      /* exponent that maps to shift 0                         */
    int64_t n_zero;     /* weights equal to +-0                                  */
    int64_t n_flushed;  /* non-zero weights below the window (incl. subnormals)  */
    int64_t n_live;     /* weights that are sampled                              */
} psbo_winfo;

/* Quantised layer as the oracle keeps it: one entry per weight, [oc][K].       */
typedef struct {
    int32_t  oc, K;         /* K = (cin/groups)*kh*kw                            */
    int8_t*  sign;          /* -1, +1; 0 = not live (zero or flushed)            */
    int32_t* shift;         /* e - e_min >= 0 for live weights                   */
    double*  p;             /* probability of the larger shift, in [0,1)         */
    int32_t  prob_bits;     /* 23: p is the full mantissa; 1..22: p is a multiple
                               of 2^-prob_bits; 1..7: samples use 7-bit uniforms  */
    psbo_winfo info;
} psbo_weights;

typedef struct { int32_t oc, cin, kh, kw, groups; } psbo_wshape;
typedef struct { int32_t n, h, w, stride_h, stride_w, pad_h, pad_w; } psbo_geom;

/* Sect. 3.1 "Value-based importance sampling", Eq. (numbersystem) and the
 * three definitions below it: s = sign(w), e = floor(log2|w|), p = |w|/2^e-1.
 * Computed on the VALUE (frexp/ldexp), not on the bit pattern.  Returns the
 * class of w; s,e,p are written for NORMAL and SUBNORMAL inputs.               */
int psbo_decode(float w, int32_t* s, int32_t* e, double* p);

/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  The paper
 * only asks that the random numbers be independent enough and uniform
 * (suppl. "Random number generation"); the counter-based generator is what
 * makes one result per (inputs, seed) well defined.                            */
void psbo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The uniform 32-bit integer of product (o,k), sample s: word (s mod 4) of
 * Philox4x32-10 with key (seed mod 2^32, seed div 2^32) and counter
 * (o, k, floor(s/4), layer_id).                                                 */
uint32_t psbo_uniform(uint64_t seed, uint32_t layer_id, uint32_t o, uint32_t k, uint32_t s);

/* The 7-bit uniform used with discretised probabilities (Sect. 4.4; suppl.
 * "Stochastic multiplier": a k_p-bit probability needs a k_p-bit comparator):
 * the low 7 bits of byte (s mod 16) of the Philox block with counter
 * (o, k, floor(s/16), layer_id); byte b of a block is bits 8*(b mod 4) .. +7 of
 * word floor(b/4).  One block serves 16 samples instead of 4.                     */
uint32_t psbo_uniform7(uint64_t seed, uint32_t layer_id, uint32_t o, uint32_t k, uint32_t s);

/* Encode a layer.  exp_bits<=0 selects 4 (Sect. 4.4: 4-bit exponents).
 * prob_bits = 23 keeps p exactly; prob_bits = 1..22 discretises it to a regular
 * grid that includes 0 and excludes 1 (Sect. 4.4): P = round-half-even(p * 2^prob_bits),
 * and P = 2^prob_bits moves the weight to the next exponent with p = 0.  A sample
 * compares P with k_p random bits (suppl. "Stochastic multiplier": a k_p-bit
 * comparator): for prob_bits = 1..7 the 7-bit uniform below (sixteen samples per
 * generator block), for prob_bits = 8..22 the top prob_bits bits of the 32-bit
 * uniform of the sample (four per block) - B = [u < P * 2^(32 - prob_bits)].  The
 * window and the overflow rule are described at the definition.  Allocates the
 * arrays of *out with malloc; release with psbo_weights_free.                   */
int  psbo_quantize(const float* w, int32_t oc, int32_t K, int32_t prob_bits, int32_t exp_bits,
                   int32_t x_absmax, int32_t s_max, psbo_weights* out);
void psbo_weights_free(psbo_weights* q);

/* Sect. 3.1, unnumbered equation after Eq. (numbersystem:simulation):
 * acc[b][oc] = sum_k sum_{s<S} sigma_k * ( x[b][k] << (shift_k + B^(s)) ).
 * u_table: optional replacement of the generator for enumeration tests,
 * u(o,k,s) = u_table[(o*K + k)*S + s] (a 32-bit uniform, or a 7-bit one when the
 * layer was encoded with prob_bits < 23); NULL = Philox.
 * overflow (nullable) receives the number of outputs whose exact (int64) sum
 * does not fit int32.                                                           */
int psbo_linear(const psbo_weights* q, const int8_t* x, int32_t B, int32_t S,
                uint64_t seed, uint32_t layer_id, const uint32_t* u_table,
                int32_t* acc, int64_t* overflow);

/* Same sum for a convolution (Sect. 3: a convolution is the same computation with
 * shared weights and a bounded support), NCHW / OIHW, with a
 * per-output-pixel sample range [from,to) (Sect. 4.5: spatially adaptive
 * sample counts whose first-pass samples are reused).
 *   budget_to   [n][oh][ow] or NULL (=> S_uniform everywhere)
 *   budget_from [n][oh][ow] or NULL (=> 0 and acc is overwritten;
 *               non-NULL => acc is read-modify-write)
 * Both maps are clamped: to' = min(to, s_max), from' = min(from, to').
 * points: optional list of n_points flat output indices; when non-NULL only
 * those outputs are computed and written to acc[0..n_points) (compact).
 * n_smac (nullable): number of sampled MACs = sum over computed outputs of
 * (to'-from') * #(live taps inside the image).                                 */
int psbo_conv2d(const psbo_weights* q, const psbo_wshape* ws, const int8_t* x,
                const psbo_geom* g, int32_t S_uniform, int32_t s_max,
                const uint8_t* budget_to, const uint8_t* budget_from,
                uint64_t seed, uint32_t layer_id,
                const int64_t* points, int64_t n_points,
                int32_t* acc, int64_t* overflow, int64_t* n_smac);

/* Shared-filter mode, Eq. (numbersystem:simulation): one binomial count per weight
 * and pass.  W[oc][k] = sigma * 2^shift * ((to-from) + B), B = number of samples
 * i in [from,to) of the stream of "output element" oc (counter (oc, k, i div 4 or
 * i div 16, layer_id)) that fall below p; 0 for weights that are not live.
 * u_table: optional replacement of the generator, u(oc,k,i) = u_table[(oc*K+k)*table_S + i].  */
int psbo_sample_filter(const psbo_weights* q, int32_t from, int32_t to, uint64_t seed,
                       uint32_t layer_id, const uint32_t* u_table, int32_t table_S, int64_t* W);

/* The layer with a filter sampled once per pass (Sect. 4.1 "Setup"; suppl.
 * "Efficient simulation of the forward pass"): acc[o] = sum_k x[o,k] * W_[from,to)[oc][k],
 * where a pixel with sample range [from,to) uses the filter built from exactly
 * those samples, so that budgets nest the way Sect. 4.5 needs (the first samples
 * are reused).  Arguments as psbo_conv2d, including the optional list of points.   */
int psbo_conv2d_shared(const psbo_weights* q, const psbo_wshape* ws, const int8_t* x,
                       const psbo_geom* g, int32_t S_uniform, int32_t s_max,
                       const uint8_t* budget_to, const uint8_t* budget_from,
                       uint64_t seed, uint32_t layer_id, const int64_t* points, int64_t n_points,
                       int32_t* acc, int64_t* overflow);

/* Final rescale: y = fl( fl( float(acc) * mult[oc] ) * inv_S ) + bias[oc],
 * every fl one binary32 round-to-nearest-even operation, no fused
 * multiply-add.  inv_S = 1/to' (0 when to' = 0).  mult NULL => 2^e_min;
 * bias NULL => no addition.  budget_to NULL => S_uniform.  spatial = oh*ow
 * (1 for a linear layer); acc is [n][oc][spatial].                              */
int psbo_rescale(const int32_t* acc, int32_t n, int32_t oc, int32_t spatial,
                 int32_t S_uniform, int32_t s_max, const uint8_t* budget_to,
                 int32_t e_min, const float* mult, const float* bias, float* y);

/* Glue between the layers of a network (suppl. "ReLU, Batch-Norm, and Pooling", "Activations and
 * Accumulation"); every floating-point step is one binary32 round-to-nearest-even operation.
 *
 * psbo_requantize: x_out[i] = clamp(rint(g(y[i] [+ r[i]]) * inv_step), lo, hi), g = max(.,0) when relu != 0,
 * r = res_f32 or (float)res_i8 * res_step (at most one of the two may be given); rint rounds ties to even.
 * psbo_maxpool_i8: NCHW max-pooling on int8, padding positions excluded (needs 2*pad <= kernel).
 * psbo_avgpool_requantize: out[n][c] = clamp(rint(((float)sum * fl(1/(h*w))) * scale), lo, hi).
 * psbo_budget_resample: nearest-pixel resampling of a budget map, source index floor(y*h/oh).          */
int psbo_requantize(const float* y, const float* res_f32, const int8_t* res_i8, float res_step,
                    int relu, float inv_step, int32_t lo, int32_t hi, int64_t n, int8_t* x_out);
int psbo_maxpool_i8(const int8_t* x, int32_t n, int32_t c, int32_t h, int32_t w, int32_t kh, int32_t kw,
                    int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int8_t* out);
int psbo_avgpool_requantize(const int8_t* x, int32_t n, int32_t c, int32_t h, int32_t w, float scale,
                            int32_t lo, int32_t hi, int8_t* out);
int psbo_budget_resample(const uint8_t* in, int32_t n, int32_t h, int32_t w, int32_t oh, int32_t ow,
                         uint8_t* out);

/* Attention mask (Sect. 4.5): entropy[n][y][x] = sum_c -softmax(a)_c log softmax(a)_c over the channels of
 * act (int8 [n][c][h][w], a = act * step), mean[n] (nullable) = mean entropy of image n, and
 * budget[n][y][x] = budget_hi where the entropy is above the image's mean, else budget_lo.  Evaluated in
 * binary64; the entropies handed out, the mean and the comparison are binary32.                        */
int psbo_attention_budget(const int8_t* act, float step, int32_t n, int32_t c, int32_t h, int32_t w,
                          uint8_t budget_lo, uint8_t budget_hi, float* entropy, float* mean, uint8_t* budget);

/* Number of host threads the layer functions spread output elements over. */
int psbo_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
