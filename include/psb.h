/*
 * psb.h -- C-ABI of the MI355X (gfx950) library for the stochastically
 * binarized scalar-product layer of Progressive Stochastic Binarization
 * (Hartmann & Wand, "Progressive Stochastic Binarization of Deep Networks").
 *
 * What the layer computes (paper, Sect. 3 and 3.1): the pre-activation
 * sum_k x_k * w_k of a linear or convolutional layer, in which every weight w
 * is replaced, for every sample, by the random power of two
 *     w_bar = s * 2^(e + B),  s = sign(w), e = floor(log2|w|),
 *     Pr(B = 1) = p = |w| / 2^e - 1                       (Eq. "numbersystem")
 * so that x * w_bar is a shift of the integer activation x, and S samples are
 * accumulated in an integer register (unnumbered equation after Eq.
 * "numbersystem:simulation"):
 *     acc = sum_k s_k * sum_{i < S} ( x_k << (e_k - e_min + B_k^(i)) ).
 * One random bit is drawn per shift (Sect. 2, last paragraph of "Hardware
 * optimized architectures"): B^(i) is independent for every (output element,
 * tap, sample).  Sample counts may differ per output pixel, and a pixel with a
 * larger count reuses the samples of the smaller one (Sect. 4.5).
 *
 * Conventions
 *  - All data pointers named *_dev are DEVICE pointers (HIP global memory of
 *    the current device); pointers named *_host are host pointers.  The caller
 *    owns every buffer; the library owns only psb_weights_t handles.
 *  - Layouts: activations NCHW int8, weights OIHW float32 (O = output channel,
 *    I = input channels per group), accumulators and outputs NCHW.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the null stream).
 *    Every call is asynchronous on that stream.  Which calls also synchronise it
 *    or allocate device memory:
 *      psb_quantize_weights     allocates the handle's memory and synchronises three
 *                               times (largest exponent, per-channel exponent
 *                               histogram, class counts);
 *      psb_weights_export       synchronous copy;
 *      per-product layer calls  (psb_linear, psb_conv2d, psb_conv2d_progressive,
 *                               psb_conv2d_requant with shared = 0) never synchronise and
 *                               never allocate, except when the channel-lane kernel cuts
 *                               the tap reduction in chunks (more than 64 taps per output,
 *                               or a layer too small to fill the chip otherwise): its
 *                               partial sums meet in scratch accumulators owned by the
 *                               handle, N*OH*OW x (OC rounded up to 64) int32, which the
 *                               first such call on a handle, and any with more outputs
 *                               than before, allocates (a growing call first synchronises
 *                               the stream and frees the old ones);
 *      shared-filter calls      allocate workspaces owned by the handle on first use and
 *                               when an input is larger than any before (then also one
 *                               synchronisation); with a budget map and no announced
 *                               levels they synchronise once to read the budget values;
 *      psb_conv2d_requant_static  never allocates, never synchronises;
 *      glue calls               never allocate, never synchronise.
 *  - Every function returns PSB_OK (0) or a negative psb_status; nothing
 *    throws, aborts or prints.  Arguments are validated on the host before any
 *    device work is started: after a NULL, SHAPE, VALUE, OVERFLOW_UNSAFE or
 *    TOO_LARGE error nothing has been launched.  A call is up to three launches
 *    (clearing, sampling, rescaling; shared-filter calls with budget maps more), so a
 *    DEVICE or ALLOC error may leave the first of them on the stream; the outputs are
 *    then unspecified.
 *  - The random bit of (output element o, tap k, sample i) is
 *        B = [ u < p * 2^32 ],
 *    u = word (i mod 4) of Philox4x32-10 with key (seed mod 2^32, seed div 2^32)
 *    and counter (o, k, i div 4, layer_id);  o is the flat NCHW index of the
 *    output element ((n*OC + oc)*OH + oy)*OW + ox (linear: b*OC + oc) and
 *    k = (ci*KH + kh)*KW + kw with ci counted inside the group.  The result is
 *    therefore a pure function of (inputs, seed, layer_id): independent of
 *    tiling, launch geometry and call order.
 *  - With probabilities discretised to prob_bits = 8..22 bits the same rule holds for the
 *    rounded p: it compares the top prob_bits bits of u [suppl. "Stochastic multiplier": a
 *    k_p-bit comparator].
 *  - With discretised probabilities of prob_bits = 1..7 bits (Sect. 4.4) p is a multiple of
 *    2^-prob_bits and a 7-bit uniform decides the bit:
 *        B = [ u7 < p * 128 ],
 *    u7 = the low 7 bits of byte (i mod 16) of the Philox block with counter
 *    (o, k, i div 16, layer_id), byte b of a block being bits 8*(b mod 4) .. +7 of
 *    word b div 4.  One generator block then serves 16 samples instead of 4.
 */
#ifndef PSB_H
#define PSB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PSB_OK = 0,
    PSB_ERR_NULL = -1,            /* a required pointer is NULL                                  */
    PSB_ERR_SHAPE = -2,           /* non-positive or inconsistent dimension                      */
    PSB_ERR_VALUE = -3,           /* NaN/Inf weight, S <= 0, S > s_max, unsupported bit width    */
    PSB_ERR_OVERFLOW_UNSAFE = -4, /* no exponent window keeps the worst case inside int32        */
    PSB_ERR_TOO_LARGE = -5,       /* N*OC*OH*OW or K does not fit the 32-bit counter words; kh or kw >= 2^15 */
    PSB_ERR_DEVICE = -6,          /* a HIP call failed; see psb_last_device_error()              */
    PSB_ERR_ALLOC = -7            /* host or device allocation failed                            */
} psb_status;

typedef struct psb_weights psb_weights_t;   /* opaque, created by psb_quantize_weights */

/* Weight tensor [oc][cin/groups][kh][kw].  A linear layer is kh = kw = groups = 1. */
typedef struct { int32_t oc, cin, kh, kw, groups; } psb_wshape;

/* Input batch and convolution geometry.  OH = (h + 2*pad_h - kh)/stride_h + 1,
 * OW likewise; no dilation.                                                        */
typedef struct { int32_t n, h, w, stride_h, stride_w, pad_h, pad_w; } psb_conv_geom;

typedef struct {
    int32_t e_top;      /* largest exponent of a normal non-zero weight             */
    int32_t e_min;      /* exponent that maps to shift 0; acc is in units 2^e_min   */
    int64_t n_zero;     /* weights equal to +-0: never sampled                      */
    int64_t n_flushed;  /* non-zero weights below the window, and subnormals        */
    int64_t n_live;     /* weights that are sampled                                 */
} psb_winfo;

/*
 * Encode a layer's weights as (sign, shift = e - e_min, 23-bit mantissa = p*2^23)
 * [Sect. 3.1, definitions of s, e, p below Eq. "numbersystem"; for a normal
 * binary32 number these are its three bit fields].
 *
 * Discretised probabilities [Sect. 4.4: probabilities on a regular grid that contains
 * p = 0 but not p = 1, because p = 1 is the next exponent]: with prob_bits = 1..22, p is
 * rounded to the nearest multiple of 2^-prob_bits, ties to the even multiple; a p that
 * rounds to 1 becomes p = 0 with e + 1.  The rounding comes first: e_top, the window and
 * the overflow rule below see the rounded weights.  A weight that rounds past the largest
 * binary32 exponent is refused (VALUE).  The exported mantissa is the rounded one.
 *
 * Exponent window [Sect. 4.4: 4-bit exponents suffice; caption of the stochastic-
 * multiplier figure: the width of the integers restricts the exponents; caption of
 * Fig. "numbersystem": too many shifts of an integer give 0]:
 * e_top = largest e in the layer; e_min = the smallest integer in
 * [e_top - (2^exp_bits - 1), e_top] such that
 *   x_absmax * s_max * max_oc sum_{k: e_k >= e_min} 2^(e_k - e_min + 1) <= 2^31 - 1,
 * which makes int32 wrap-around impossible for |x| <= x_absmax and up to s_max
 * samples.  Weights below e_min, subnormals and zeros are not live.
 *
 *  w_dev      device, float32 [oc][cin/groups][kh][kw], read only during the call
 *  prob_bits  23 (p exact: the full binary32 mantissa), 8..22 (rounded p, still one 32-bit uniform per
 *             sample) or 1..7 (rounded p, sixteen 7-bit uniforms per generator block)
 *  exp_bits   1..5; <= 0 selects 4
 *  x_absmax   1..128, largest |activation| the caller will pass
 *  s_max      1..255, largest sample count / budget the caller will use
 *  out        receives the handle (device memory owned by the library)
 * Errors: NULL, SHAPE, VALUE (NaN/Inf weight, bad widths, rounded out of range), OVERFLOW_UNSAFE,
 * TOO_LARGE, DEVICE, ALLOC.
 */
int psb_quantize_weights(const float* w_dev, const psb_wshape* shape, int32_t prob_bits, int32_t exp_bits,
                         int32_t x_absmax, int32_t s_max, void* hip_stream, psb_weights_t** out);

/* Copy the summary of the encoding to *info (host). */
int psb_weights_info(const psb_weights_t* q, psb_winfo* info);

/* Copy the encoded weights to host memory: packed_host[oc*K + k] =
 * sign<<31 | shift<<23 | mantissa, with shift = 0xFF for a weight that is not live.
 * Synchronous. */
int psb_weights_export(const psb_weights_t* q, uint32_t* packed_host);

/* Release a handle (NULL is allowed).  The caller must make sure no layer call
 * using it is still running.
 * A handle also owns a device word with which the layer kernel hands out work to its
 * workgroups (every call resets it on its stream before the kernel starts) and the
 * workspaces named below.  Layer calls that use the SAME handle must therefore not
 * overlap in time (same stream, or ordered by events); calls on different handles may
 * run concurrently. */
void psb_weights_destroy(psb_weights_t* q);

/* Output height/width of a convolution, on the host, with the validation every
 * conv entry point applies (SHAPE, TOO_LARGE).  oh/ow may be NULL. */
int psb_conv2d_out_dims(const psb_wshape* shape, const psb_conv_geom* geom, int32_t* oh, int32_t* ow);

/*
 * Linear layer [Sect. 3, Eq. 1, with every product replaced per Sect. 3.1]:
 *   acc[b][oc] = sum_{k live} sigma_k * sum_{i<S} ( x[b][k] << (shift_k + B(o,k,i)) ),  o = b*OC + oc.
 *  x_dev    device, int8 [B][K], K = cin
 *  acc_dev  device, int32 [B][OC], overwritten
 *  y_dev    device, float32 [B][OC] or NULL.  y = fl(fl(float(acc) * mult[oc]) * fl(1/S)) + bias[oc],
 *           every fl one binary32 round-to-nearest operation, no fused multiply-add
 *           [the ">> n" normalisation of the shift form, Sect. 3.1; the affine map of a
 *           folded batch normalisation, Sect. 3, Eq. 2]
 *  mult_dev device, float32 [OC] or NULL (= 2^e_min for every channel)
 *  bias_dev device, float32 [OC] or NULL (= no addition)
 * Errors: NULL, SHAPE, VALUE (S <= 0 or S > s_max), TOO_LARGE, DEVICE.
 */
int psb_linear(const psb_weights_t* q, const int8_t* x_dev, int32_t B, int32_t S, uint64_t seed,
               uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev,
               const float* bias_dev, void* hip_stream);

/*
 * Convolution with the same sample count S at every output [Sect. 3: a convolution is the
 * same computation with shared weights and a bounded support; otherwise as psb_linear].  Taps that fall
 * into the padding contribute 0 and are not sampled.
 *  x_dev    device, int8 [N][C][H][W]
 *  acc_dev  device, int32 [N][OC][OH][OW], overwritten
 *  y_dev, mult_dev, bias_dev as in psb_linear, shaped [N][OC][OH][OW] / [OC].
 */
int psb_conv2d(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom, int32_t S,
               uint64_t seed, uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev,
               const float* bias_dev, void* hip_stream);

/*
 * Convolution with a per-output-pixel sample range [Sect. 4.5: a low-precision pass
 * everywhere, more samples only where needed, the first samples being reused].
 * Pixel (n,oy,ox), all output channels alike, draws samples from'..to'-1 with
 *   to' = min(budget_to, s_max), from' = min(budget_from, to')   (0 if budget_from is NULL).
 *  budget_to_dev    device, uint8 [N][OH][OW]
 *  budget_from_dev  device, uint8 [N][OH][OW] or NULL.
 *                   NULL: acc is overwritten.  Non-NULL: acc is read-modify-write; it must
 *                   hold the result of samples 0..from'-1 of the same (seed, layer_id), and
 *                   afterwards holds the result of samples 0..to'-1, bit-identical to a
 *                   single call with budget_from NULL.
 *  y_dev            uses fl(1/to') per pixel (0 where to' = 0).
 */
int psb_conv2d_progressive(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom,
                           const uint8_t* budget_to_dev, const uint8_t* budget_from_dev, uint64_t seed,
                           uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev,
                           const float* bias_dev, void* hip_stream);

/*
 * Shared-filter mode [Eq. "numbersystem:simulation": w -> s 2^e (B_{n,p}/n + 1), one binomial count per
 * WEIGHT and pass; Sect. 4.1 "Setup" and suppl. "Efficient simulation of the forward pass": the filter is
 * sampled directly, then the layer is an ordinary convolution].  This is the granularity every accuracy
 * figure of the paper was measured with; it is a different (cheaper, spatially correlated) estimator from
 * the per-product mode of the entry points above and gives different bits.  In integers:
 *     W[oc][k] = sigma * 2^shift * ((to - from) + B),  B = #{ i in [from,to) : uniform(oc, k, i) decides 1 },
 *     acc[o]   = sum_k x[o,k] * W[oc][k]               (exact: the overflow rule of the encoding covers it)
 * where uniform(oc, k, i) is the stream the per-product mode gives to output element o := oc.
 * The contraction runs on the int8 matrix cores for groups = 1 and on a direct kernel otherwise.
 *
 * psb_sample_filter writes W for samples [sample_from, sample_to) to w_dev (device, int32 [OC][K], 0 for
 * weights that are not live).  Errors: NULL, VALUE (empty or negative range, sample_to > s_max), DEVICE.
 *
 * psb_linear_shared / psb_conv2d_shared / psb_conv2d_progressive_shared take the arguments of their
 * per-product namesakes and return acc and y in the same units (y = acc * 2^e_min / n_samples [+ bias]).
 * With a budget map, a pixel with range [from', to') uses the filter built from exactly those samples, so
 * a refinement call adds what the first call left out [Sect. 4.5].
 * Differences from the per-product calls: the first shared-filter call on a handle, and any call with a
 * larger input than before, allocates device memory owned by the handle (the sampled filter, its int8
 * digit planes, a channels-last copy of the activations); psb_conv2d_progressive_shared synchronises the
 * stream once (it reads back which budget values occur).  Additional errors: TOO_LARGE when
 * kh*kw*(cin rounded up to 32) >= 2^17 (groups = 1) or when the channels-last activation tensor
 * (n*h*w*(cin rounded up to 32) bytes) reaches 2 GiB, which the matrix-core kernel's 32-bit offsets
 * cannot address; ALLOC.
 */
int psb_sample_filter(const psb_weights_t* q, int32_t sample_from, int32_t sample_to, uint64_t seed,
                      uint32_t layer_id, int32_t* w_dev, void* hip_stream);
int psb_linear_shared(const psb_weights_t* q, const int8_t* x_dev, int32_t B, int32_t S, uint64_t seed,
                      uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev,
                      const float* bias_dev, void* hip_stream);
int psb_conv2d_shared(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom, int32_t S,
                      uint64_t seed, uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev,
                      const float* bias_dev, void* hip_stream);
int psb_conv2d_progressive_shared(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom,
                                  const uint8_t* budget_to_dev, const uint8_t* budget_from_dev, uint64_t seed,
                                  uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev,
                                  const float* bias_dev, void* hip_stream);

/*
 * Glue between the layers of a network [suppl. "ReLU, Batch-Norm, and Pooling": ReLU is a gate on the
 * sign bit, max-pooling needs comparators, the factor of an average pooling can be a fixed multiplication;
 * suppl. "Activations and Accumulation": activations are stored as fixed-point integers].  The affine map of
 * a folded batch normalisation is the mult/bias of the layer calls.  All pointers are device pointers; the
 * calls are asynchronous on hip_stream.  Every floating-point step is one binary32 round-to-nearest-even
 * operation in the order written, so the integers do not depend on compiler or launch shape.
 *
 * psb_requantize: layer output to the next layer's activations,
 *     x[i] = clamp( rint( g( y[i] [+ r[i]] ) * inv_step ), lo, hi ),   rint: ties to even,
 *     g = max(., 0) if relu != 0 (NaN -> 0), else identity;
 *     r = res_f32[i], or (float)res_i8[i] * res_step (one rounded multiplication); at most one of the two
 *     residual operands may be non-NULL (VALUE otherwise); -128 <= lo <= hi <= 127 and inv_step >= 0 (VALUE
 *     otherwise); n > 0 elements.
 * psb_maxpool2d_i8: NCHW int8 max-pooling; positions in the padding do not take part; needs 2*pad <= kernel
 *     (SHAPE otherwise).  out is [n][c][OH][OW] with the OH/OW rule of psb_conv_geom.
 * psb_maxpool2d_i8_blocked: the same pooling on the blocked channels-last layout, x = [n][h][ceil(c/32)][w][32] and
 *     out = [n][OH][ceil(c/32)][OW][32] (both 16-byte aligned, VALUE otherwise); the padding channels of a block are
 *     pooled like the others (whatever they hold), so a chain of layers stays in this layout from the first
 *     convolution on.
 * psb_global_avgpool_requantize: out[n][c] = clamp( rint( ((float)sum * fl(1/(h*w))) * scale ), lo, hi ),
 *     sum = exact integer sum over the h*w positions (h*w <= 2^23).
 * psb_budget_resample: a budget map at another resolution [Sect. 4.5: the two kinds of regions are applied
 *     to the activations of every layer], out[n][y][x] = in[n][floor(y*h/oh)][floor(x*w/ow)].
 */
/* A layer call with psb_requantize fused into its epilogue: the next layer's activations leave the kernel that
 * produced the accumulators, without a round trip of the fp32 values through memory.
 *   x_out[o] = clamp( rint( g( y[o] [+ r[o]] ) * inv_step ), lo, hi )  with y as defined for psb_linear and
 *   g, r, rint exactly as in psb_requantize (residual operands are indexed like the output, [N][OC][OH][OW]).
 * budget_to_dev NULL: S samples everywhere; non-NULL: the per-pixel budget map of psb_conv2d_progressive
 * (no refinement form).  shared != 0 selects the shared-filter mode.  A linear layer is geometry {B,1,1,1,1,0,0}.
 * y_dev may be NULL, and so may acc_dev: then no accumulators are handed out (a network pass does not read
 * them), which saves their write; where a kernel combines partial sums in the accumulators the library uses
 * scratch memory owned by the handle instead (allocated on first use, grown on demand).
 * Errors: those of the layer call, plus NULL (rq, x_out_dev), VALUE (two residual operands, bad clamp range)
 * (also a negative or NaN inv_step) and ALLOC. */
typedef struct {
    int32_t relu;                 /* != 0: g = max(., 0)                                */
    float inv_step;
    int32_t lo, hi;               /* -128 <= lo <= hi <= 127                            */
    const float* res_f32_dev;     /* at most one of the two residual operands, or none */
    const int8_t* res_i8_dev;
    float res_step;
} psb_requant;
int psb_conv2d_requant(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom, int32_t S,
                       const uint8_t* budget_to_dev, uint64_t seed, uint32_t layer_id, int32_t* acc_dev,
                       float* y_dev, const float* mult_dev, const float* bias_dev, const psb_requant* rq,
                       int8_t* x_out_dev, int32_t shared, void* hip_stream);

/*
 * psb_conv2d_requant for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  It is psb_conv2d_requant with acc_dev = NULL and shared = 0 (per-product
 * mode, requantised activations and/or rescaled values out, no accumulators handed out), element for element, but
 * the scratch memory of its kernels - the ticket counter of the persistent layer kernel and the accumulators in
 * which the partial sums of a split tap reduction meet - is a fixed array inside the library's device code instead
 * of memory owned by the handle.  The call issues no hipMalloc, no hipFree and no synchronisation.
 *  - Limit: n * OH * OW * (oc rounded up to a multiple of 64) <= PSB_STATIC_MAX_OUTPUTS (the array holds that many
 *    int32 accumulators, 32 MiB, plus 256 bytes; each GPU the library runs on holds it until the process ends).
 *    Larger calls return TOO_LARGE and launch nothing.
 *  - All calls on one GPU share that GPU's array, and it keeps the last call's contents; the call clears what it
 *    needs (in a kernel, not a memset, so it can be captured).  Two such calls that overlap in time on one GPU -
 *    different streams without ordering - race on it; same-stream calls are ordered and safe.
 *  - The array's device address is looked up once per GPU, by psb_quantize_weights (any handle of that GPU), which
 *    therefore has to have run outside the capture - it allocates and synchronises anyway.
 * Errors: those of psb_conv2d_requant without ALLOC, plus TOO_LARGE as above.
 */
#define PSB_STATIC_MAX_OUTPUTS (8 * 1024 * 1024)
int psb_conv2d_requant_static(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom, int32_t S,
                              const uint8_t* budget_to_dev, uint64_t seed, uint32_t layer_id, float* y_dev,
                              const float* mult_dev, const float* bias_dev, const psb_requant* rq, int8_t* x_out_dev,
                              void* hip_stream);

/*
 * The chained shared-filter pass [Sect. 4.1 and suppl. "Efficient simulation of the forward pass": one sampled
 * filter per layer and pass].  Two additions for callers that run layer after layer on one GPU:
 *
 * Blocked channels-last activations.  The matrix-core kernel reads its int8 activations as
 *     xb[ (((n * H + y) * CB + c / 32) * W + x) * 32 + c % 32 ],   CB = ceil(C / 32)
 * (blocks of 32 channels, the pixels of a row contiguous; padding channels are ignored on input and
 * unspecified on output).  psb_conv2d_shared_requant_blocked is psb_conv2d_requant with shared = 1, a uniform S,
 * no accumulator output, and `layout` saying which of its int8 tensors use that layout: PSB_BLOCKED_IN (x_dev:
 * read in place, no copy is made), PSB_BLOCKED_OUT (x_out_dev), PSB_BLOCKED_RES (rq->res_i8_dev); the others, and
 * the fp32 tensors, are [N][C][H][W].  y_dev and x_out_dev are both optional but not both NULL; with x_out_dev NULL
 * rq is not read (a shortcut branch: only the rescaled values).  Results are those of psb_conv2d_requant, element
 * for element.
 * Blocked tensors must be 16-byte (input) / 4-byte (output, residual) aligned (VALUE otherwise).  PSB_BLOCKED_IN
 * needs a layer that runs on the matrix cores (groups = 1) with more than 32 / kw input channels (SHAPE otherwise:
 * such layers - a network's first - take [N][C][H][W]).
 *
 * psb_shared_prepare_filters samples the digit planes of n handles in one launch, for S samples and the given
 * (seed, layer_id) of each.  The next shared-filter call on such a handle with the same S, seed and layer_id and
 * no budget map uses them instead of sampling again (once: the call after that samples as usual); any other
 * shared-filter call on the handle discards them.  Handles whose layers do not run on the matrix cores are
 * skipped.  The call counts as a layer call on every handle it is given (it writes their workspaces) and must not
 * overlap with other calls on them.  handles, seeds and layer_ids are host arrays of n entries.  Same results as
 * without the call.  Errors: NULL, SHAPE (n <= 0), VALUE (S), DEVICE, TOO_LARGE, ALLOC.
 * Errors of psb_conv2d_shared_requant_blocked: those of psb_conv2d_requant, plus VALUE (unknown layout bits,
 * alignment) and SHAPE (PSB_BLOCKED_IN on a layer that cannot take it).
 */
enum { PSB_BLOCKED_IN = 1, PSB_BLOCKED_OUT = 2, PSB_BLOCKED_RES = 4 };
int psb_conv2d_shared_requant_blocked(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom, int32_t S,
                                      uint64_t seed, uint32_t layer_id, float* y_dev, const float* mult_dev,
                                      const float* bias_dev, const psb_requant* rq, int8_t* x_out_dev, int32_t layout,
                                      void* hip_stream);
int psb_shared_prepare_filters(const psb_weights_t* const* handles, int32_t n, int32_t S, const uint64_t* seeds,
                               const uint32_t* layer_ids, void* hip_stream);

/*
 * The second pass of the two-stage scheme as a chain [Sect. 4.5: more samples only inside the mask, on all layers,
 * the first samples reused].  psb_conv2d_shared_budget_requant_blocked is psb_conv2d_shared_requant_blocked with a
 * per-pixel budget map instead of one S, and the budget values of the pass given with the call:
 *  budget_to_dev  device, uint8 [N][OH][OW]
 *  levels_host    host array of n_levels budget values (any order, duplicates and zeros ignored, each clamped to
 *                 s_max); at most four distinct values (VALUE otherwise).
 * A pixel's budget is rounded DOWN to the largest listed value it reaches (0 if it reaches none: such a pixel gets
 * no sample, y = bias); the result is, element for element, what psb_conv2d_requant (shared = 1) gives for the map
 * rounded that way.  The levels l_1 < l_2 < ... cut the sample axis into the nested segments [0, l_1), [l_1, l_2),
 * ..., each with its own sampled filter; on the matrix cores all segments run in ONE launch - a tile accumulates
 * the contractions of the segments its pixels reach in the same registers, then the fused epilogue - with no
 * read-back, no synchronisation, no zero-fill and no separate rescale launch, so the call can be captured into a
 * HIP graph.  Layers that do not run that way (groups > 1, a reduction that is split over the grid) take the
 * segments one launch at a time on a rounded copy of the map, with the same results.
 * psb_shared_prepare_filters_levels samples the filters of all segments of n handles in one launch (two when there
 * are more than 32 filters); the next psb_conv2d_shared_budget_requant_blocked call on such a handle with the same
 * levels, seed and layer_id uses them, once.
 * Errors: those of psb_conv2d_shared_requant_blocked, plus NULL (budget_to_dev, levels_host), SHAPE (n_levels
 * outside 1..256), VALUE (more than four distinct levels; prepare: no level above 0).
 */
int psb_conv2d_shared_budget_requant_blocked(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom,
                                             const uint8_t* budget_to_dev, const uint8_t* levels_host, int32_t n_levels,
                                             uint64_t seed, uint32_t layer_id, float* y_dev, const float* mult_dev,
                                             const float* bias_dev, const psb_requant* rq, int8_t* x_out_dev,
                                             int32_t layout, void* hip_stream);
int psb_shared_prepare_filters_levels(const psb_weights_t* const* handles, int32_t n, const uint8_t* levels_host,
                                      int32_t n_levels, const uint64_t* seeds, const uint32_t* layer_ids, void* hip_stream);

/* Budget values of the NEXT call, told in advance [Sect. 4.5: the two-stage scheme has two].  A shared-filter call
 * with a budget map (psb_conv2d_progressive_shared, psb_conv2d_requant with shared = 1) cuts the sample axis at
 * every value that occurs in the map; by default it finds those values itself, which costs a read-back and a stream
 * synchronisation.  After psb_shared_budget_levels(levels, n) the calling thread's next such call - that one call
 * only - takes the n values of the host array `levels` instead (clamped to the handle's s_max; 0 is added when there
 * is no budget_from map) and issues no synchronisation.  EVERY value that occurs in that call's maps (budget_to and
 * budget_from, after clamping) must be among them: a pixel whose budget is missing receives the samples of the next
 * lower listed value only while its result is still divided by its own budget.  (psb_conv2d_shared_budget_requant_blocked
 * takes the levels as an argument and rounds budgets down to them instead.)  Listed values that do not occur cost
 * one filter sampling and one empty launch each.  n = 0 (levels may be NULL) withdraws an announcement.  Host only.
 * Errors: NULL (n > 0 without levels), SHAPE (n < 0 or n > 256). */
int psb_shared_budget_levels(const uint8_t* levels_host, int32_t n);

int psb_requantize(const float* y_dev, const float* res_f32_dev, const int8_t* res_i8_dev, float res_step,
                   int32_t relu, float inv_step, int32_t lo, int32_t hi, int64_t n, int8_t* x_dev, void* hip_stream);
int psb_maxpool2d_i8(const int8_t* x_dev, int32_t n, int32_t c, int32_t h, int32_t w, int32_t kh, int32_t kw,
                     int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int8_t* out_dev,
                     void* hip_stream);
int psb_maxpool2d_i8_blocked(const int8_t* x_dev, int32_t n, int32_t c, int32_t h, int32_t w, int32_t kh, int32_t kw,
                             int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int8_t* out_dev,
                             void* hip_stream);
int psb_global_avgpool_requantize(const int8_t* x_dev, int32_t n, int32_t c, int32_t h, int32_t w, float scale,
                                  int32_t lo, int32_t hi, int8_t* out_dev, void* hip_stream);
int psb_budget_resample(const uint8_t* in_dev, int32_t n, int32_t h, int32_t w, int32_t oh, int32_t ow,
                        uint8_t* out_dev, void* hip_stream);

/*
 * Attention mask [Sect. 4.5: the pixelwise entropy of the softmax over the channels of the last
 * convolutional layer, h_xy = sum_c -softmax(a_xyc) log softmax(a_xyc), with a hard threshold at the mean
 * entropy of the image; the regions above the mean get the larger sample count].
 *  act_dev      int8 [n][c][h][w], a = act * step (step > 0)
 *  entropy_dev  float32 [n][h][w], written (evaluated in binary64 with the device library's exp/log, rounded once)
 *  mean_dev     float32 [n] or NULL: mean entropy of each image (binary64 sum in a fixed order, rounded once)
 *  budget_dev   uint8 [n][h][w]: budget_hi where entropy > mean (strictly), else budget_lo
 * The map can be handed to psb_conv2d_progressive at the resolution of any layer via psb_budget_resample.
 * Errors: NULL, SHAPE, VALUE (step not positive and finite), DEVICE.
 */
int psb_attention_budget(const int8_t* act_dev, float step, int32_t n, int32_t c, int32_t h, int32_t w,
                         uint8_t budget_lo, uint8_t budget_hi, float* entropy_dev, float* mean_dev,
                         uint8_t* budget_dev, void* hip_stream);

/* The hipError_t (as int) of the last failed HIP call on this thread, 0 if none. */
int psb_last_device_error(void);

/* Identifies the sources the library was built from: the hexadecimal SHA-256 of the concatenated source files
 * (this header and the files under csrc/, in the order the build script lists them), as given to the compiler by
 * the build script; "unknown" for a build made any other way.  The Python binding refuses to load a library whose
 * identifier differs from the hash of the sources beside it.  The pointer is valid for the life of the process. */
const char* psb_build_id(void);

/* Select the kernel mapping for subsequent layer calls of this process:
 * 0 = automatic, 1 = one output pixel per lane (any layer; the simplest kernel), 2 = one output
 * channel per lane (groups = 1 only; made for dense layers), 3 = compacted product list per
 * (channel, 256 pixels) (any layer; made for grouped, depthwise and pruned layers).
 * Results are bit-identical for every mapping; the switch exists for tests and benchmarks.
 * Shared-filter calls: 1 selects their direct kernel for every layer, any other value leaves the
 * choice (matrix cores for groups = 1) to the library.
 * Returns the previous value. */
int psb_set_mapping(int mapping);

/* The mapping (1, 2 or 3) a layer call with this handle and geometry would run with under the
 * current psb_set_mapping value; negative psb_status on invalid arguments (NULL, SHAPE,
 * TOO_LARGE; SHAPE also when mapping 2 is forced on a grouped layer).  Host only: no device work. */
int psb_query_mapping(const psb_weights_t* q, const psb_conv_geom* geom);

/* Shared-filter mode, host only (no device work; for tests): the number of 16-byte slots per half plane that the
 * 3 x 3 kernel with both operands in LDS reserves for the input window of one pixel tile (128 * half_tiles consecutive
 * output pixels, half_tiles = 1 or 2) of a layer with this geometry - an upper bound on
 *     vpos(last pixel) - vpos(first pixel) + 2 (w + 1) + 3,   vpos(n, oy, ox) = (n (h + 1) + oy) (w + 1) + ox,
 * over all tiles and batch sizes - or 0 when that kernel does not take the geometry (not 3 x 3 / stride 1 / padding 1,
 * or more than 512 slots) and the call runs in the plain matrix-core kernel.  SHAPE for non-positive sizes. */
int psb_shared_window_slots(int32_t kh, int32_t kw, const psb_conv_geom* geom, int32_t half_tiles);

/* Timing of the sampling kernels, for benchmarks.  While enabled, every layer call
 * brackets its sampling kernel (not the zero-fill or the separate rescale kernel) with a
 * pair of HIP events on the caller's stream; at most 4096 pairs are kept between reads.
 * psb_profile_read waits for the recorded events, adds up their elapsed times, returns
 * the sum in milliseconds and the number of launches, and clears the record.  Not
 * thread-safe; enable/disable only while no layer call is in flight. */
int psb_profile_enable(int on);
int psb_profile_read(double* kernel_ms_sum, int64_t* n_launches);

#ifdef __cplusplus
}
#endif
#endif
