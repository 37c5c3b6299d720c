// Device kernels of the PSB layer library (gfx950, wave64).
//
//  - weight encoding: exponent scan, per-channel exponent histogram, packing
//  - "pixel-lane" layer kernel: one output element per lane, one output channel per
//    workgroup; works for every layer shape (groups, strides, pruned weights)
//
// The packed weight word is  sign<<31 | shift<<23 | mantissa(23 bit);  a weight that is
// not sampled (zero, subnormal, below the exponent window) has shift = 0xFF.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "psb_philox.hip.h"

namespace psb {

constexpr uint32_t kDeadWord = 0x7F800000u;  // shift field 0xFF, nothing else
constexpr int kHistBins = 32;                // exponent window is at most 2^5 wide

// ---------------------------------------------------------------------------------
// Weight encoding (Sect. 3.1: s = sign w, e = floor(log2|w|), p = |w|/2^e - 1; for a
// normal binary32 these are its sign bit, exponent field - 127 and mantissa / 2^23).
// ---------------------------------------------------------------------------------

// Discretised probabilities (Sect. 4.4): p is rounded, ties to even, to a multiple of 2^-prob_bits;
// the grid holds 0 but not 1, so a p that rounds to 1 becomes p = 0 at the next exponent.  On the bit
// pattern this is one integer addition into the exponent|mantissa field, whose carry does the exponent
// step.  A weight pushed past the largest finite exponent comes out with the exponent field of an
// infinity and is reported like one.  Zeros, subnormals, NaN and Inf are returned unchanged.
__device__ __forceinline__ uint32_t round_probability(uint32_t bits, int prob_bits)
{
    const uint32_t f = (bits >> 23) & 0xFFu;
    if (prob_bits >= 23 || f == 0u || f == 0xFFu) return bits;
    const int drop = 23 - prob_bits;
    const uint32_t em = bits & 0x7FFFFFFFu;
    const uint32_t q = em >> drop;
    const uint32_t rem = em & ((1u << drop) - 1u);
    const uint32_t half = 1u << (drop - 1);
    const uint32_t up = (rem > half || (rem == half && (q & 1u))) ? 1u : 0u;
    return (bits & 0x80000000u) | ((q + up) << drop);
}

// scan[0] = largest exponent field among normal non-zero weights after rounding (0 if none)
// scan[1] = 1 if any weight is NaN or Inf, or is rounded past the largest finite exponent
__global__ void __launch_bounds__(256) k_exponent_scan(const uint32_t* __restrict__ w_bits, int64_t n,
                                                       int prob_bits, uint32_t* __restrict__ scan)
{
    uint32_t best = 0, bad = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t f = (round_probability(w_bits[i], prob_bits) >> 23) & 0xFFu;
        if (f == 0xFFu) bad = 1;
        else if (f > best) best = f;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        best = max(best, (uint32_t)__shfl_xor((int)best, off, 64));
        bad |= (uint32_t)__shfl_xor((int)bad, off, 64);
    }
    // one pair of atomics per workgroup: thousands of waves hitting the same word serialise
    __shared__ uint32_t s_best[4], s_bad[4];
    if ((threadIdx.x & 63) == 0) { s_best[threadIdx.x >> 6] = best; s_bad[threadIdx.x >> 6] = bad; }
    __syncthreads();
    if (threadIdx.x == 0) {
        best = max(max(s_best[0], s_best[1]), max(s_best[2], s_best[3]));
        bad = s_bad[0] | s_bad[1] | s_bad[2] | s_bad[3];
        if (best) atomicMax(&scan[0], best);
        if (bad) atomicOr(&scan[1], 1u);
    }
}

// hist[oc][b] = number of normal weights of channel oc whose exponent is e_top - b,
// b = 0 .. window.  One workgroup per output channel.
__global__ void __launch_bounds__(256) k_exponent_hist(const uint32_t* __restrict__ w_bits, int K, int prob_bits,
                                                       int field_top, int window, uint32_t* __restrict__ hist)
{
    __shared__ uint32_t bins[kHistBins];
    if (threadIdx.x < kHistBins) bins[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t* row = w_bits + (int64_t)blockIdx.x * K;
    for (int k = threadIdx.x; k < K; k += blockDim.x) {
        const int f = (int)((round_probability(row[k], prob_bits) >> 23) & 0xFFu);
        const int b = field_top - f;
        if (f != 0 && b >= 0 && b <= window) atomicAdd(&bins[b], 1u);
    }
    __syncthreads();
    if (threadIdx.x < kHistBins) hist[(int64_t)blockIdx.x * kHistBins + threadIdx.x] = bins[threadIdx.x];
}

// packed[oc][k] (row-major, the export format) and tile[k][oc_pad] (transposed, padded
// with dead entries to a multiple of 64 channels, for the channel-lane kernel):
// tile entry = { threshold,  unit = +-2^shift (0 when not live) }; the threshold is mantissa << 9 for
// 32-bit uniforms (prob_bits 8..23: the mantissa is exact or rounded to prob_bits bits, and the comparison with
// the 32-bit uniform is a comparison of its top prob_bits bits) and the 7-bit numerator of p in each of the four
// bytes for 7-bit uniforms (prob_bits 1..7).
// counts[0..2] = zero, flushed, live.
__device__ __forceinline__ uint32_t threshold_of(uint32_t mant, int prob_bits)
{
    return prob_bits <= 7 ? (mant >> 16) * 0x01010101u : mant << 9;
}

__global__ void __launch_bounds__(256) k_pack(const uint32_t* __restrict__ w_bits, int OC, int K, int oc_pad,
                                              int prob_bits, int field_min /* exponent field of e_min */,
                                              uint32_t* __restrict__ packed, uint2* __restrict__ tile,
                                              unsigned long long* __restrict__ counts)
{
    // One workgroup per 64 channels x 64 taps: the weights are read and `packed` is written along k (both
    // [oc][K]), the words go through LDS, and `tile` is written along oc ([k][oc_pad]): every access coalesced.
    __shared__ uint32_t words[64][64 + 1];
    const int k0 = blockIdx.x * 64, oc0 = blockIdx.y * 64;
    unsigned long long n_zero = 0, n_flush = 0, n_live = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int idx = r * 256 + threadIdx.x;
        const int oc = oc0 + (idx >> 6), k = k0 + (idx & 63);
        uint32_t word = kDeadWord;
        if (oc < OC && k < K) {
            const uint32_t bits = round_probability(w_bits[(int64_t)oc * K + k], prob_bits);
            const int f = (int)((bits >> 23) & 0xFFu);
            const uint32_t mant = bits & 0x7FFFFFu;
            if (f == 0 && mant == 0) n_zero++;
            else if (f == 0 || f < field_min) n_flush++;
            else {
                n_live++;
                word = (bits & 0x80000000u) | ((uint32_t)(f - field_min) << 23) | mant;
            }
            packed[(int64_t)oc * K + k] = word;
        }
        words[idx >> 6][idx & 63] = word;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int idx = r * 256 + threadIdx.x;
        const int k = k0 + (idx >> 6), oc = oc0 + (idx & 63);       // oc < oc_pad: oc_pad is a multiple of 64
        if (k < K) {
            const uint32_t word = words[idx & 63][idx >> 6];
            uint2 entry = make_uint2(0u, 0u);
            if ((word & 0x7F800000u) != kDeadWord) {
                const uint32_t unit = 1u << ((word >> 23) & 0xFFu);          // shift <= 30 by the overflow rule
                entry = make_uint2(threshold_of(word & 0x7FFFFFu, prob_bits), (word & 0x80000000u) ? (0u - unit) : unit);
            }
            tile[(int64_t)k * oc_pad + oc] = entry;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        n_zero += __shfl_xor(n_zero, off, 64);
        n_flush += __shfl_xor(n_flush, off, 64);
        n_live += __shfl_xor(n_live, off, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        if (n_zero) atomicAdd(&counts[0], n_zero);
        if (n_flush) atomicAdd(&counts[1], n_flush);
        if (n_live) atomicAdd(&counts[2], n_live);
    }
}

// ---------------------------------------------------------------------------------
// Layer kernels
// ---------------------------------------------------------------------------------

// Optional second output of a layer call: the next layer's 8-bit activations, made from the rescaled value in
// the same kernel (suppl. "ReLU, Batch-Norm, and Pooling": ReLU as a gate on the sign; "Activations and
// Accumulation": fixed-point activations):  x = clamp(rint(g(y [+ r]) * inv_step), lo, hi).
struct Requant {
    int8_t* x_out;            // null: no fused requantisation
    const float* res_f32;     // residual operand, or null
    const int8_t* res_i8;     // residual operand as integers times res_step, or null
    float res_step, inv_step, lo, hi;
    int relu;
    // Layout of x_out / of res_i8: 0 = [N][OC][OH][OW]; 1 = blocked channels-last [N][OH][ceil(OC/32)][OW][32]
    // (the layout the shared-filter kernel reads its activations in).  res_f32 is always [N][OC][OH][OW].
    int out_blocked, res_blocked;
};

struct LayerParams {
    // tensors
    const uint32_t* packed;    // [OC][K]
    const uint2* tile;         // [K][oc_pad] {threshold, unit}
    const int8_t* x;           // [N][C][H][W]
    const uint8_t* budget_to;  // [N][OH][OW] or null
    const uint8_t* budget_from;  // [N][OH][OW] or null (non-null: acc is read-modify-write)
    int32_t* acc;              // [N][OC][OH][OW]
    int32_t* acc_cl;           // channel-lane kernel with a split tap reduction: partial sums [N*OH*OW][oc_pad]
    float* y;                  // same shape or null
    const float* mult;         // [OC] or null
    const float* bias;         // [OC] or null
    // geometry
    int N, C, H, W, OC, OH, OW, KH, KW, Cg, OCg, K, oc_pad;
    int stride_h, stride_w, pad_h, pad_w;
    // sampling
    int S, s_max;
    int prob_bits;             // 8..23: 32-bit uniforms, 4 per generator block; 1..7: 7-bit uniforms, 16 per block
    uint32_t key0, key1, layer_id;
    float default_mult;        // 2^e_min
    int max_shift;             // largest shift of a live weight
    Requant rq;
};

// Number of samples i in [from,to) of product (o,k) whose uniform is below thr.
// Block j of the generator serves samples 4j .. 4j+3.
__device__ __forceinline__ uint32_t count_below(uint32_t o, uint32_t k, uint32_t layer, uint32_t key0,
                                                uint32_t key1, uint32_t thr, int from, int to)
{
    uint32_t n = 0;
    for (int j = from >> 2; 4 * j < to; ++j) {
        const u32x4 r = philox4x32_10(u32x4{o, k, (uint32_t)j, layer}, key0, key1);
        const int s0 = 4 * j;
        n += (s0 + 0 >= from && s0 + 0 < to && r.x < thr) ? 1u : 0u;
        n += (s0 + 1 >= from && s0 + 1 < to && r.y < thr) ? 1u : 0u;
        n += (s0 + 2 >= from && s0 + 2 < to && r.z < thr) ? 1u : 0u;
        n += (s0 + 3 >= from && s0 + 3 < to && r.w < thr) ? 1u : 0u;
    }
    return n;
}

// 7-bit uniforms (Sect. 4.4: a k_p-bit probability needs k_p random bits per sample): sample i of a
// product is the low 7 bits of byte i mod 16 of generator block i div 16, bytes numbered from the
// least significant byte of word 0.  thr4 holds the 7-bit threshold in each byte.
//
// Bytes of one word whose 7-bit uniform is NOT below the threshold, among the bytes selected by
// valid (0x80 in each selected byte): with bit 7 forced to one no byte borrows from its neighbour,
// and bit 7 of (0x80 + u) - t survives exactly when u >= t.
__device__ __forceinline__ uint32_t not_below7(uint32_t word, uint32_t thr4, uint32_t valid)
{
    return (uint32_t)__popc(((word | 0x80808080u) - thr4) & valid);
}

// 0x80 in byte b of word w of block j for every sample 16j + 4w + b inside [from, to)
__device__ __forceinline__ uint32_t valid_bytes7(int j, int w, int from, int to)
{
    const int base = 16 * j + 4 * w;
    const int lo = min(max(from - base, 0), 4), hi = min(max(to - base, 0), 4);
    const uint32_t below_hi = hi >= 4 ? 0xFFFFFFFFu : (1u << (8 * hi)) - 1u;
    const uint32_t below_lo = lo >= 4 ? 0xFFFFFFFFu : (1u << (8 * lo)) - 1u;
    return below_hi & ~below_lo & 0x80808080u;
}

// Number of samples i in [from,to) of product (o,k) whose 7-bit uniform is below the threshold.
__device__ __forceinline__ uint32_t count_below7(uint32_t o, uint32_t k, uint32_t layer, uint32_t key0,
                                                 uint32_t key1, uint32_t thr4, int from, int to)
{
    uint32_t not_below = 0;
    for (int j = from >> 4; 16 * j < to; ++j) {
        const u32x4 r = philox4x32_10(u32x4{o, k, (uint32_t)j, layer}, key0, key1);
        not_below += not_below7(r.x, thr4, valid_bytes7(j, 0, from, to));
        not_below += not_below7(r.y, thr4, valid_bytes7(j, 1, from, to));
        not_below += not_below7(r.z, thr4, valid_bytes7(j, 2, from, to));
        not_below += not_below7(r.w, thr4, valid_bytes7(j, 3, from, to));
    }
    return (uint32_t)(to - from) - not_below;
}

// Workgroups are dealt to the 8 XCDs of the chip round-robin by their linear index, and every XCD has its own L2.
// For a grid whose x size is a multiple of 8, this maps workgroup index b (XCD b mod 8, the (b div 8)-th workgroup
// of that XCD) to one of n work items so that every XCD gets a contiguous range, the ranges differing in length
// by at most one; 0xFFFFFFFF for the surplus workgroups of an XCD with a shorter range.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned b, unsigned n)
{
    const unsigned xcd = b & 7u, local = b >> 3;
    const unsigned begin = (unsigned)(((uint64_t)xcd * n) >> 3), end = (unsigned)(((uint64_t)(xcd + 1u) * n) >> 3);
    return begin + local < end ? begin + local : 0xFFFFFFFFu;
}

// Final rescale: four separately rounded binary32 operations.
__device__ __forceinline__ float rescale(int32_t acc, float mult, int to, const float* bias, int oc)
{
    const float inv_s = (to > 0) ? __fdiv_rn(1.0f, (float)to) : 0.0f;
    float r = __fmul_rn(__fmul_rn(__int2float_rn(acc), mult), inv_s);
    if (bias) r = __fadd_rn(r, bias[oc]);
    return r;
}

// clamp(rint(v), lo, hi) as an integer; NaN goes to lo
__device__ __forceinline__ int32_t round_clamp(float v, float lo, float hi)
{
    float q = rintf(v);               // v_rndne_f32: ties to even
    if (!(q >= lo)) q = lo;
    if (q > hi) q = hi;
    return (int32_t)q;
}

__device__ __forceinline__ int32_t requantize_one(float y, bool has_res, float r, bool relu, float inv_step, float lo,
                                                  float hi)
{
    float t = y;
    if (has_res) t = __fadd_rn(t, r);
    if (relu && !(t > 0.0f)) t = 0.0f;
    return round_clamp(__fmul_rn(t, inv_step), lo, hi);
}

// Everything a layer kernel writes besides the accumulator: the rescaled value and/or the requantised activation
// of output element o (channel oc, `to` samples).  P is LayerParams or the shared-filter mode's parameter block.
// Index of output element o = ((n * OC + oc) * OH + oy) * OW + ox in the blocked channels-last layout.
template <class P>
__device__ __forceinline__ int64_t blocked_index(const P& p, int64_t o, int oc)
{
    const int64_t hw = (int64_t)p.OH * p.OW;
    const int64_t n = o / (hw * p.OC);
    const int pix = (int)(o % hw);
    const int oy = pix / p.OW, ox = pix - oy * p.OW;
    return ((((n * p.OH + oy) * ((p.OC + 31) >> 5) + (oc >> 5)) * p.OW + ox) << 5) + (oc & 31);
}

template <class P>
__device__ __forceinline__ void emit(const P& p, int64_t o, int oc, int32_t acc, int to)
{
    if (!p.y && !p.rq.x_out) return;
    const float r = rescale(acc, p.mult ? p.mult[oc] : p.default_mult, to, p.bias, oc);
    if (p.y) p.y[o] = r;
    if (p.rq.x_out) {
        const int64_t ob = (p.rq.out_blocked || p.rq.res_blocked) ? blocked_index(p, o, oc) : o;
        float res = 0.0f;
        if (p.rq.res_f32) res = p.rq.res_f32[o];
        if (p.rq.res_i8) res = __fmul_rn((float)p.rq.res_i8[p.rq.res_blocked ? ob : o], p.rq.res_step);
        p.rq.x_out[p.rq.out_blocked ? ob : o] = (int8_t)requantize_one(r, p.rq.res_f32 || p.rq.res_i8, res, p.rq.relu != 0,
                                                                       p.rq.inv_step, p.rq.lo, p.rq.hi);
    }
}

// One output element per lane; blockIdx.y = output channel, so the weight word and the
// tap position are wave-uniform (scalar loads, scalar branches on dead weights) and the
// activation reads of neighbouring lanes are neighbouring bytes.
__global__ void __launch_bounds__(256) k_layer_pixel_lane(const LayerParams p)
{
    const int oc = blockIdx.y;
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    const int64_t pix = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pix >= npix) return;
    const int ox = (int)(pix % p.OW);
    const int oy = (int)((pix / p.OW) % p.OH);
    const int n = (int)(pix / ((int64_t)p.OW * p.OH));

    int to = p.budget_to ? (int)p.budget_to[pix] : p.S;
    to = min(to, p.s_max);
    int from = p.budget_from ? (int)p.budget_from[pix] : 0;
    from = min(from, to);

    const uint32_t o = (uint32_t)((((int64_t)n * p.OC + oc) * p.OH + oy) * p.OW + ox);
    const int grp = oc / p.OCg;
    const uint32_t* wrow = p.packed + (int64_t)oc * p.K;
    const int8_t* xn = p.x + ((int64_t)n * p.C + (int64_t)grp * p.Cg) * p.H * p.W;
    const int iy0 = oy * p.stride_h - p.pad_h;
    const int ix0 = ox * p.stride_w - p.pad_w;

    int32_t acc = 0;
    if (to > from) {
        int k = 0;
        for (int ci = 0; ci < p.Cg; ++ci) {
            for (int kh = 0; kh < p.KH; ++kh) {
                for (int kw = 0; kw < p.KW; ++kw, ++k) {
                    const uint32_t word = wrow[k];
                    if ((word & 0x7F800000u) == kDeadWord) continue;
                    const int iy = iy0 + kh, ix = ix0 + kw;
                    if (iy < 0 || iy >= p.H || ix < 0 || ix >= p.W) continue;
                    const int32_t xv = xn[((int64_t)ci * p.H + iy) * p.W + ix];
                    if (xv == 0) continue;
                    const uint32_t thr = threshold_of(word & 0x7FFFFFu, p.prob_bits);
                    const uint32_t cnt = p.prob_bits <= 7
                        ? count_below7(o, (uint32_t)k, p.layer_id, p.key0, p.key1, thr, from, to)
                        : count_below(o, (uint32_t)k, p.layer_id, p.key0, p.key1, thr, from, to);
                    const int32_t shifted = (int32_t)((uint32_t)xv << ((word >> 23) & 0xFFu));
                    const int32_t term = shifted * (int32_t)((uint32_t)(to - from) + cnt);
                    acc += (word & 0x80000000u) ? -term : term;
                }
            }
        }
    }
    if (p.budget_from) acc += p.acc[o];
    if (p.acc) p.acc[o] = acc;          // null: the caller only wants the requantised activations
    emit(p, o, oc, acc, to);
}

}  // namespace psb
