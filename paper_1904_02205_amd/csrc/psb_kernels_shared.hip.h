// Shared-filter mode (Eq. "numbersystem:simulation"; Sect. 4.1 "Setup"; suppl. "Efficient simulation of the
// forward pass"): one binomial count per WEIGHT and per pass, then an ordinary integer convolution with the
// sampled filter
//     W[oc][k] = sigma * 2^shift * ((to - from) + B),   B = #{ i in [from,to) : u(oc, k, i) < threshold }.
// The random stream of weight (oc, k) is the per-product stream of "output element" oc.
//
// With a filter shared by all pixels the layer IS a dense contraction, so it runs on the int8 matrix cores:
//   * W (up to 31 bits + sign) is split into up to four balanced base-256 digits d_b in [-128,127],
//     W = sum_b d_b 256^b (mod 2^32); each digit plane is contracted separately with
//     v_mfma_i32_32x32x32_i8 and the planes are recombined with shifts in the epilogue.  All of it is exact
//     modulo 2^32, and the true result fits int32 by the overflow rule of the weight encoding.
//   * the activations are read in a blocked channels-last layout [N][H][C/32][W][32] (a copy made by the
//     prologue launch, or the caller's tensor if it already has that layout): the 16 bytes of reduction index a
//     lane feeds to the matrix core are 16 consecutive bytes, and the 32 pixels of a half tile are 1 KB of
//     consecutive memory; the reduction index is ordered (kh, kw, channel), which no result depends on;
//   * the digit planes are written directly in the operand order of the instruction
//     [block of 32 channels][k-step][plane][lane][16 bytes]: an operand is one coalesced 1 KB read.
// One wave computes 32 output channels x 64 (or 32) output pixels.  Three kernels share the pieces below: the
// plain one (weights staged through LDS chunk by chunk), a persistent one for short reductions (all weights of a
// channel block resident in LDS) and the direct one for grouped layers.
//
// Per-pixel budgets: the distinct budget values cut the sample axis into segments; each segment is one
// filter (built from exactly its samples, so budgets nest) and one masked, accumulating contraction over
// the pixels whose range contains the segment.
//
// Grouped and depthwise layers have no contraction worth a matrix core (a depthwise channel has 9 taps):
// they use a direct kernel on the int32 filter.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "psb_kernels.hip.h"

namespace psb {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kPlaneStride = 64 * 16;   // bytes of one operand (64 lanes x 16 bytes)
constexpr int kMaxPlanes = 4;

struct SharedParams {
    const int8_t* x;           // [N][C][H][W]                      (direct kernel)
    const int8_t* xt;          // [N][H][C_pad/32][W][32]: blocks of 32 channels, pixels of a row contiguous (matrix-core kernel)
    const int8_t* planes;      // [OC/32][n_ksteps][4][64][16]
    const int32_t* w32;        // [OC][K]
    const uint8_t* budget_to;  // [N][OH][OW] or null
    const uint8_t* budget_from;
    int32_t* acc;
    float* y;
    const float* mult;
    const float* bias;
    int N, C, H, W, OC, OH, OW, KH, KW, Cg, OCg, K, C_pad, n_ksteps;
    int stride_h, stride_w, pad_h, pad_w;
    int S, s_max;
    uint32_t xt_bytes;         // size of xt (below 2^31): operand loads are range-checked against it
    // Geometry of the convolution as the matrix-core kernel sees it on xt.  Normally the layer's own; for layers
    // with very few input channels (kw * C <= 32) xt holds, per output column, the kw x C values of one kernel row
    // ("row packing"), and the kernel sees a kh x 1 convolution with unit column stride on an image OW wide.
    int tH, tW, tKH, tKW, t_stride_h, t_stride_w, t_pad_h, t_pad_w;
    int ksplit;                // the reduction is cut into ksplit parts (grid z); > 1: results are added atomically
    int masked;                // 0: every pixel, acc overwritten, epilogue fused.  1: only pixels whose sample
    int seg_from, seg_to;      //    range contains [seg_from, seg_to); acc accumulated
    // Budget map with announced levels, in one launch (n_seg > 0; masked = 0, budget_to given, no budget_from):
    // levels l_1 < ... < l_n cut the sample axis into nested segments [l_(i-1), l_i), l_0 = 0, each with its own
    // sampled filter (digit planes seg_stride bytes apart).  A pixel's budget is rounded DOWN to a level (0 if it is
    // below all of them); the pixel takes part in segment i when that level is >= l_i.  The segments' contractions
    // accumulate in the same registers (a pixel that does not take part feeds zeros), and the epilogue is fused.
    int n_seg;
    int seg_level[4];
    uint64_t seg_stride;
    float default_mult;
    // floor(2^32 / d) for d = OW, OH, tW + 1, tH + 1 (inverse_of): the matrix-core kernels decompose pixel indices with
    // a multiplication instead of a division (some 30 instructions each, per half tile and per pixel tile)
    uint32_t inv_OW, inv_OH, inv_W1, inv_H1;
    // k_conv3x3_window: 1 = each XCD works on an eighth of the CHANNEL blocks (all pixel tiles) instead of an eighth of
    // the pixel tiles (all channel blocks) - for layers whose weights outweigh their activations (set by the launcher)
    int xcd_by_channels;
    Requant rq;
    // [N][OC][OH][OW] byte tensors of the fused requantisation move as 32-bit words (four pixels of one channel,
    // after a byte transpose over four lanes) when OH * OW and the tensor's address are multiples of 4:
    int quad_store;            // ... x_out
    int quad_res;              // ... res_i8
};

// Filter sampling: count and filter value of one weight; digit planes for the matrix cores.
struct FilterJob {
    const uint32_t* packed;   // [OC][K]
    int OC, K, KHW, CB, n_ksteps, prob_bits, from, to;
    int pack_KW, pack_C;      // row packing: kernel width and channel count (0: not packed)
    int n_planes;             // digit planes the contraction of this sample range reads
    int C;                    // input channels (K / KHW)
    uint32_t inv_ksteps, inv_CB, inv_pack_C;   // floor(2^32 / d) of the three divisors of the index arithmetic
    uint32_t key0, key1, layer_id;
    int32_t* w32;             // [OC][K], or null when only the planes are wanted
    int8_t* planes;           // operand-ordered digit planes, or null
};

// The ten pairs of round keys of a generator key: uniform over a job, so they are computed once per wave and kept
// in scalar registers instead of being stepped inside every generator call.
struct RoundKeys { uint32_t k0[10], k1[10]; };
__device__ __forceinline__ RoundKeys round_keys(uint32_t key0, uint32_t key1)
{
    RoundKeys rk;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        rk.k0[r] = key0 + (uint32_t)r * kWeyl0;
        rk.k1[r] = key1 + (uint32_t)r * kWeyl1;
    }
    return rk;
}

// count_below() for the whole generator blocks 0 .. NB - 1 of one weight (samples 0 .. 4 NB - 1): no per-sample
// range tests, and what the blocks share is computed once - in round 0 the product with the output index, in round 1
// the product with state word 2 (neither depends on the block number, whose own product is a constant).
template <int NB>
__device__ __forceinline__ uint32_t count_below_blocks(uint32_t o, uint32_t k, uint32_t layer, const RoundKeys& rk, uint32_t thr)
{
    uint32_t hi_a, lo_a, hi_b1, lo_b1;
    mulhilo(kMulA, o, hi_a, lo_a);
    const uint32_t z1 = hi_a ^ layer ^ rk.k1[0];               // state word 2 after round 0
    mulhilo(kMulB, z1, hi_b1, lo_b1);
    uint32_t n = 0;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        uint32_t hi_bj, lo_bj, hi_a1, lo_a1;
        mulhilo(kMulB, (uint32_t)j, hi_bj, lo_bj);             // constants
        const uint32_t x1 = hi_bj ^ k ^ rk.k0[0];              // state after round 0: (x1, lo_bj, z1, lo_a)
        mulhilo(kMulA, x1, hi_a1, lo_a1);
        u32x4 c{hi_b1 ^ lo_bj ^ rk.k0[1], lo_b1, hi_a1 ^ lo_a ^ rk.k1[1], lo_a1};      // after round 1
#pragma unroll
        for (int r = 2; r < 10; ++r) c = philox_round(c, rk.k0[r], rk.k1[r]);
        n += (c.x < thr ? 1u : 0u) + (c.y < thr ? 1u : 0u) + (c.z < thr ? 1u : 0u) + (c.w < thr ? 1u : 0u);
    }
    return n;
}

// W[oc][k] for the job's sample range, from the weight's encoded word.  whole_blocks: 1..4 when the range is samples
// 0 .. 4 whole_blocks - 1 of 32-bit uniforms (the usual call), else 0; rk: round_keys() of the job's key.
__device__ __forceinline__ int32_t sample_word(const FilterJob& j, uint32_t word, int oc, int k, int whole_blocks = 0,
                                               const RoundKeys* rk = nullptr)
{
    if ((word & 0x7F800000u) == kDeadWord) return 0;
    const uint32_t thr = threshold_of(word & 0x7FFFFFu, j.prob_bits);
    uint32_t cnt;
    if (whole_blocks == 1) cnt = count_below_blocks<1>((uint32_t)oc, (uint32_t)k, j.layer_id, *rk, thr);
    else if (whole_blocks == 2) cnt = count_below_blocks<2>((uint32_t)oc, (uint32_t)k, j.layer_id, *rk, thr);
    else if (whole_blocks == 3) cnt = count_below_blocks<3>((uint32_t)oc, (uint32_t)k, j.layer_id, *rk, thr);
    else if (whole_blocks == 4) cnt = count_below_blocks<4>((uint32_t)oc, (uint32_t)k, j.layer_id, *rk, thr);
    else cnt = j.prob_bits <= 7
        ? count_below7((uint32_t)oc, (uint32_t)k, j.layer_id, j.key0, j.key1, thr, j.from, j.to)
        : count_below((uint32_t)oc, (uint32_t)k, j.layer_id, j.key0, j.key1, thr, j.from, j.to);
    const uint32_t mag = ((uint32_t)(j.to - j.from) + cnt) << ((word >> 23) & 0xFFu);   // < 2^31 by the overflow rule
    return (word & 0x80000000u) ? -(int32_t)mag : (int32_t)mag;
}

// One thread per weight: the int32 filter.
__device__ __forceinline__ void sample_filter_thread(const FilterJob& j, int64_t i)
{
    if (i >= (int64_t)j.OC * j.K) return;
    const int oc = (int)(i / j.K);
    j.w32[i] = sample_word(j, j.packed[i], oc, (int)(i - (int64_t)oc * j.K));
}

// 4 x 4 byte transpose across the four lanes of a quad: afterwards byte i of lane j is what byte j of
// lane i was.  Every lane of the quad must be active.
__device__ __forceinline__ uint32_t quad_transpose_bytes(uint32_t d)
{
    const uint32_t d0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)d, 0x00, 0xF, 0xF, true);   // quad_perm [0,0,0,0]
    const uint32_t d1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)d, 0x55, 0xF, 0xF, true);   // [1,1,1,1]
    const uint32_t d2 = (uint32_t)__builtin_amdgcn_mov_dpp((int)d, 0xAA, 0xF, 0xF, true);   // [2,2,2,2]
    const uint32_t d3 = (uint32_t)__builtin_amdgcn_mov_dpp((int)d, 0xFF, 0xF, 0xF, true);   // [3,3,3,3]
    // byte j of d0, d1 into bytes 0, 1 and byte j of d2, d3 into bytes 2, 3 (selector byte 0x0c yields zero)
    const uint32_t j = threadIdx.x & 3u;
    const uint32_t lo = __builtin_amdgcn_perm(d1, d0, 0x0c0c0000u | ((4u + j) << 8) | j);
    const uint32_t hi = __builtin_amdgcn_perm(d3, d2, 0x00000c0cu | ((4u + j) << 24) | (j << 16));
    return lo | hi;
}

// x / d and x % d for any 32-bit x, given inv = floor(2^32 / d) (0xFFFFFFFF for d = 1): the product's high word
// is the quotient or one less.
__host__ __device__ inline uint32_t inverse_of(uint32_t d) { return d <= 1u ? 0xFFFFFFFFu : (uint32_t)(0x100000000ull / d); }
__device__ __forceinline__ uint32_t div_mod(uint32_t x, uint32_t d, uint32_t inv, uint32_t& rem)
{
    uint32_t q = __umulhi(x, inv);
    uint32_t r = x - q * d;
    if (r >= d) { ++q; r -= d; }
    rem = r;
    return q;
}

// Digit planes in operand order: one thread per (channel, slot) of a 32-channel x 32-slot operand block, padding
// included (those get zeros, so the buffer needs no clearing), and kPlaneGroup operand blocks per thread, so that
// the weight words of all of them are in flight before the first is sampled.  Workgroup `block` of the job works
// on operand blocks (block >> 2) * kPlaneGroup + g, each = (channel block, reduction step) - uniform values, whose
// divisions run on the scalar unit - and its thread t' = (block & 3) * 256 + thread index on slot (bits 0-3 and
// 9 of t') of channel (bits 4-8).  The four lanes of a quad hold four consecutive slots; after the byte transpose
// lane b of the quad stores plane b's four digits as one 32-bit word.
constexpr int kPlaneGroup = 4;

__device__ __forceinline__ void sample_planes_block(const FilterJob& j, uint32_t block)
{
    const uint32_t t = (block & 3u) * 256u + threadIdx.x;
    const int cl = (int)(t & 15u) + 16 * (int)((t >> 9) & 1u);
    const int ocl = (int)(t >> 4) & 31;
    const uint32_t n_blk = (uint32_t)((j.OC + 31) >> 5) * (uint32_t)j.n_ksteps;
    const uint32_t blk0 = (block >> 2) * kPlaneGroup;
    uint32_t word[kPlaneGroup];
    int oc_[kPlaneGroup], k_[kPlaneGroup];
    bool valid[kPlaneGroup];
#pragma unroll
    for (int g = 0; g < kPlaneGroup; ++g) {
        const uint32_t blk = min(blk0 + g, n_blk - 1);     // past the end: the last block again (not stored)
        uint32_t kstep;
        const uint32_t ocb = div_mod(blk, (uint32_t)j.n_ksteps, j.inv_ksteps, kstep);
        const int oc = (int)ocb * 32 + ocl;
        int c, r;
        bool ok = oc < j.OC;
        if (j.pack_KW) {                               // one step per kernel row; slot kw * C + c inside it
            uint32_t cu;
            const int kw = (int)div_mod((uint32_t)cl, (uint32_t)j.pack_C, j.inv_pack_C, cu);
            c = (int)cu;
            r = (int)kstep * j.pack_KW + kw;
            ok = ok && kw < j.pack_KW;
        } else {
            uint32_t cb;
            r = (int)div_mod(kstep, (uint32_t)j.CB, j.inv_CB, cb);
            c = (int)cb * 32 + cl;
            ok = ok && c < j.C;
        }
        oc_[g] = oc;
        k_[g] = c * j.KHW + r;
        valid[g] = ok;
        word[g] = ok ? j.packed[(int64_t)oc * j.K + k_[g]] : kDeadWord;
    }
    const int plane = (int)(t & 3);
    const RoundKeys rk = round_keys(j.key0, j.key1);
    const int whole_blocks = (j.prob_bits > 7 && j.from == 0 && (j.to & 3) == 0 && j.to <= 16) ? j.to >> 2 : 0;   // uniform
#pragma unroll
    for (int g = 0; g < kPlaneGroup; ++g) {
        // Balanced base-256 digits d_b in [-128, 127] with v = sum d_b 256^b modulo 2^32, all four at once: adding 128
        // to every digit gives the ordinary digits (0..255) of v + 0x80808080, and subtracting 128 from a byte
        // flips its top bit.
        const uint32_t v = valid[g] ? (uint32_t)sample_word(j, word[g], oc_[g], k_[g], whole_blocks, &rk) : 0u;
        const uint32_t digits = (v + 0x80808080u) ^ 0x80808080u;
        const uint32_t out = quad_transpose_bytes(digits);
        if (plane < j.n_planes && blk0 + g < n_blk)
            *reinterpret_cast<uint32_t*>(j.planes + (((int64_t)(blk0 + g) * kMaxPlanes + plane) * 64 + ocl + 32 * (cl >> 4)) * 16 +
                                         (cl & 12)) = out;
    }
}

// x [N][C][H][W] -> xt [N][H][C_pad/32][W][32] (zeros in the padding channels).  One workgroup per tile of
// 32 channels x 64 consecutive positions of an image plane, transposed through LDS.
struct TransposeJob {
    const int8_t* x;
    int C, H, W, C_pad;
    int8_t* xt;
    int N;
    int tiles_p;          // tiles per image plane: ceil(H * W / 64), or / 256 with `wide`
    int wide;             // H * W and the address of x are multiples of 4: the copy moves 32-bit words
    int64_t rows;         // N * H
    // row packing (pack_KW > 0): xt[n][iy][ox][kw * C + c] = x[n][c][iy][ox * stride_w - pad_w + kw], zero outside
    // the row and in the unused slots; one thread per (n, iy, ox)
    int pack_KW, OW, stride_w, pad_w;
};

__device__ __forceinline__ void row_pack_block(const TransposeJob& j, int64_t block)
{
    const int64_t i = block * 256 + threadIdx.x;          // (n * H + iy) * OW + ox
    if (i >= j.rows * j.OW) return;
    const uint32_t i32 = (uint32_t)i;                     // rows * OW is below 2^31 (xt has 32 bytes per element)
    const uint32_t row = i32 / (uint32_t)j.OW;
    const int ox = (int)(i32 - row * (uint32_t)j.OW);
    const int n = (int)(row / (uint32_t)j.H), iy = (int)(row - (uint32_t)n * (uint32_t)j.H);
    const int ix0 = ox * j.stride_w - j.pad_w;
    // All 32 slots in straight-line code: slot s = kw * C + c; a slot outside the row (or beyond kw * C) reads
    // element 0 of the tensor instead and is masked, so the loads do not wait for each other.
    const uint32_t plane = (uint32_t)(j.H * j.W);
    const uint32_t base = ((uint32_t)n * (uint32_t)j.C * (uint32_t)j.H + (uint32_t)iy) * (uint32_t)j.W;   // x[n][0][iy][0]
    const int n_slots = j.pack_KW * j.C;
    uint32_t v[32];
    int kw = 0, c = 0;                                    // uniform, stepped on the scalar unit
#pragma unroll
    for (int s = 0; s < 32; ++s) {
        const int ix = ix0 + kw;
        const bool ok = (s < n_slots) & ((unsigned)ix < (unsigned)j.W);
        const uint32_t at = ok ? base + (uint32_t)c * plane + (uint32_t)ix : 0u;
        const uint32_t b = (uint8_t)j.x[at];
        v[s] = ok ? b : 0u;
        if (++c == j.C) { c = 0; ++kw; }
    }
    uint32_t w[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) w[q] = v[4 * q] | (v[4 * q + 1] << 8) | (v[4 * q + 2] << 16) | (v[4 * q + 3] << 24);
    uint4* dst = reinterpret_cast<uint4*>(j.xt + i * 32);
    dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
    dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
}

__device__ __forceinline__ void channels_last_tile(const TransposeJob& j, int64_t tile_index, int8_t (*tile)[64 + 4])
{
    // tile = 32 channels x 64 consecutive positions of one image plane (positions run over rows, so that narrow
    // images still fill the tile); tiles of a plane first, then images, then channel blocks
    const uint32_t plane = (uint32_t)(j.H * j.W);
    const uint32_t p0 = (uint32_t)(tile_index % j.tiles_p) * 64u;
    const int n = (int)((tile_index / j.tiles_p) % j.N);
    const int c0 = (int)(tile_index / ((int64_t)j.tiles_p * j.N)) * 32;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int idx = r * 256 + threadIdx.x;
        const int c = idx >> 6;
        const uint32_t pos = p0 + (uint32_t)(idx & 63);
        int8_t v = 0;
        if (c0 + c < j.C && pos < plane) v = j.x[((int64_t)n * j.C + c0 + c) * plane + pos];
        tile[c][idx & 63] = v;
    }
    __syncthreads();
    const int dx = threadIdx.x >> 2, part = threadIdx.x & 3;
    const uint32_t pos = p0 + (uint32_t)dx;
    if (pos < plane) {
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            lo |= (uint32_t)(uint8_t)tile[part * 8 + q][dx] << (8 * q);
            hi |= (uint32_t)(uint8_t)tile[part * 8 + 4 + q][dx] << (8 * q);
        }
        const uint32_t iy = pos / (uint32_t)j.W, ix = pos - iy * (uint32_t)j.W;
        const int64_t row = (int64_t)n * j.H + iy;
        uint2* dst = reinterpret_cast<uint2*>(j.xt + (((row * (j.C_pad >> 5) + (c0 >> 5)) * j.W + ix) * 32 + part * 8));
        *dst = make_uint2(lo, hi);
    }
}

// The same copy for image planes whose size and address are multiples of 4 bytes (TransposeJob::wide): a tile is
// 32 channels x 256 consecutive plane positions.  A thread loads four positions of four channels as four 32-bit
// words (a wave reads 256 consecutive bytes of each channel), transposes the 4 x 4 bytes in registers and writes
// four words of four channels each into a position-major LDS tile; after the barrier it owns one position and
// moves its 32 channel bytes with two 16-byte reads and two 16-byte stores.
constexpr int kWideTilePositions = 256;
constexpr int kWideTileRow = 48;            // bytes per position in LDS: 32 used, padded to spread the banks
__device__ __forceinline__ void channels_last_tile_wide(const TransposeJob& j, int64_t tile_index, int8_t* tile)
{
    const uint32_t plane = (uint32_t)(j.H * j.W);
    const uint32_t p0 = (uint32_t)(tile_index % j.tiles_p) * (uint32_t)kWideTilePositions;
    const int n = (int)((tile_index / j.tiles_p) % j.N);
    const int c0 = (int)(tile_index / ((int64_t)j.tiles_p * j.N)) * 32;
    uint32_t w[2][4];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int unit = r * 256 + (int)threadIdx.x;       // (channel quad, position quad)
        const int cq = unit >> 6;
        const uint32_t pos = p0 + 4u * (uint32_t)(unit & 63);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = c0 + cq * 4 + i;
            w[r][i] = 0;
            if (c < j.C && pos < plane)
                w[r][i] = *reinterpret_cast<const uint32_t*>(j.x + ((int64_t)n * j.C + c) * plane + pos);
        }
    }
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int unit = r * 256 + (int)threadIdx.x;
        const int cq = unit >> 6, pq = unit & 63;
        // byte b of w[r][i] = channel i, position b  ->  byte i of out[b]
        const uint32_t t0 = __builtin_amdgcn_perm(w[r][1], w[r][0], 0x05010400u);
        const uint32_t t1 = __builtin_amdgcn_perm(w[r][3], w[r][2], 0x05010400u);
        const uint32_t t2 = __builtin_amdgcn_perm(w[r][1], w[r][0], 0x07030602u);
        const uint32_t t3 = __builtin_amdgcn_perm(w[r][3], w[r][2], 0x07030602u);
        const uint32_t out[4] = {__builtin_amdgcn_perm(t1, t0, 0x05040100u), __builtin_amdgcn_perm(t1, t0, 0x07060302u),
                                 __builtin_amdgcn_perm(t3, t2, 0x05040100u), __builtin_amdgcn_perm(t3, t2, 0x07060302u)};
#pragma unroll
        for (int b = 0; b < 4; ++b)
            *reinterpret_cast<uint32_t*>(tile + (pq * 4 + b) * kWideTileRow + cq * 4) = out[b];
    }
    __syncthreads();
    const uint32_t pos = p0 + threadIdx.x;
    if (pos < plane) {
        const uint4 lo = *reinterpret_cast<const uint4*>(tile + (int)threadIdx.x * kWideTileRow);
        const uint4 hi = *reinterpret_cast<const uint4*>(tile + (int)threadIdx.x * kWideTileRow + 16);
        const uint32_t iy = pos / (uint32_t)j.W, ix = pos - iy * (uint32_t)j.W;
        const int64_t row = (int64_t)n * j.H + iy;
        uint4* dst = reinterpret_cast<uint4*>(j.xt + ((row * (j.C_pad >> 5) + (c0 >> 5)) * j.W + ix) * 32);
        dst[0] = lo;
        dst[1] = hi;
    }
}

// The digit planes of several layers in one launch (a network pass samples all its filters at once): job i owns
// the workgroups [first_block[i], first_block[i + 1]); entries past the last job hold 0xFFFFFFFF.
constexpr int kMaxBatchJobs = 32;
struct FilterBatch {
    FilterJob jobs[kMaxBatchJobs];
    unsigned first_block[kMaxBatchJobs + 1];
};

__global__ void __launch_bounds__(256) k_sample_planes_batch(const FilterBatch b)
{
    // the job of this workgroup = number of later jobs' first workgroups it has reached; without a loop over
    // dependent loads (the table arrives in a few wide scalar loads, the rest is scalar compares)
    int i = 0;
#pragma unroll
    for (int k = 1; k < kMaxBatchJobs; ++k) i += (blockIdx.x >= b.first_block[k]) ? 1 : 0;
    sample_planes_block(b.jobs[i], blockIdx.x - b.first_block[i]);
}

__global__ void __launch_bounds__(256) k_sample_filter(const FilterJob j)
{
    sample_filter_thread(j, (int64_t)blockIdx.x * 256 + threadIdx.x);
}

// Both preparations of a shared-filter call in one launch: workgroups [0, filter_blocks) sample the filter,
// the rest transpose the activations.  The two jobs are independent of each other.
__global__ void __launch_bounds__(256) k_shared_prologue(const FilterJob f, const TransposeJob t, unsigned filter_blocks)
{
    __shared__ __align__(16) int8_t tile[kWideTilePositions * kWideTileRow];
    if (blockIdx.x < filter_blocks) {        // uniform over the workgroup
        if (f.planes) sample_planes_block(f, blockIdx.x);
        else sample_filter_thread(f, (int64_t)blockIdx.x * 256 + threadIdx.x);
    } else if (t.pack_KW)
        row_pack_block(t, (int64_t)(blockIdx.x - filter_blocks));
    else if (t.wide)
        channels_last_tile_wide(t, (int64_t)(blockIdx.x - filter_blocks), tile);
    else
        channels_last_tile(t, (int64_t)(blockIdx.x - filter_blocks), reinterpret_cast<int8_t(*)[64 + 4]>(tile));
}

// present[v] = 1 for every clamped budget value v that occurs in the maps
__global__ void __launch_bounds__(256) k_budget_levels(const uint8_t* __restrict__ budget_to,
                                                       const uint8_t* __restrict__ budget_from, int64_t npix, int s_max,
                                                       uint32_t* __restrict__ present)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < npix; i += (int64_t)gridDim.x * blockDim.x) {
        const int to = min((int)budget_to[i], s_max);
        const int from = budget_from ? min((int)budget_from[i], to) : 0;
        present[to] = 1u;
        present[from] = 1u;
    }
}

// out[i] = the largest of the n ascending levels that min(in[i], s_max) reaches, 0 if it reaches none
struct BudgetLevels { int n; int level[4]; };
__global__ void __launch_bounds__(256) k_budget_round_down(const uint8_t* __restrict__ in, int64_t npix, int s_max,
                                                           const BudgetLevels lv, uint8_t* __restrict__ out)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < npix; i += (int64_t)gridDim.x * blockDim.x) {
        const int to = min((int)in[i], s_max);
        int eff = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (k < lv.n && lv.level[k] <= to) eff = lv.level[k];
        out[i] = (uint8_t)eff;
    }
}

// sample range of a pixel and whether it takes part in this launch
__device__ __forceinline__ bool shared_pixel_range(const SharedParams& p, int64_t pix, int& to)
{
    to = p.budget_to ? (int)p.budget_to[pix] : p.S;
    to = min(to, p.s_max);
    if (p.n_seg > 0) {                 // the largest announced level that the budget reaches
        int eff = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i < p.n_seg && p.seg_level[i] <= to) eff = p.seg_level[i];
        to = eff;
    }
    if (!p.masked) return true;
    int from = p.budget_from ? (int)p.budget_from[pix] : 0;
    from = min(from, to);
    return from <= p.seg_from && p.seg_to <= to;
}

// Operand movement.  The four waves of a workgroup work on the same block of 32 output channels, so the
// weight operands are staged through LDS, kStageSteps reduction steps at a time, and shared: the next
// chunk is already on its way into registers while the current one is consumed.  The activation operands
// differ per wave and come straight from global memory (the few input rows a tile touches stay in L1/L2)
// through a software pipeline: the operands of step s + kDepth are requested right after step s has been
// consumed.  Every load is unconditional, so that nothing but the matrix instructions waits on memory.
// Activation operands are fetched with range-checked buffer loads: a tap in the padding gets an offset beyond the
// buffer and the hardware returns zeros for it, so every load is unconditional and no zero-filled memory is needed.
constexpr uint32_t kOutOfRange = 0x80000000u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t operand_buffer(const int8_t* base, uint32_t bytes)
{
    // raw buffer (stride 0): the record count is in bytes; 0x00020000 = 32-bit data format, as gfx9 wants it
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(base), 0, (int)bytes, 0x00020000);
}

// 16 bytes at base + lane_offset + uniform_offset, zeros when lane_offset is outside the buffer
__device__ __forceinline__ v4i load_operand(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_offset, uint32_t uniform_offset)
{
    typedef unsigned int v4u __attribute__((ext_vector_type(4)));
    const v4u v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)lane_offset, (int)uniform_offset, 0);
    return v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
}

constexpr int kDepth = 4;
constexpr int kStageSteps = 8;      // a multiple of kDepth

// Load cursor of a wave: the reduction step whose activation operands are requested next.  Steps are ordered
// (kh, kw, block of 32 channels); step, position and the two offsets are uniform over the wave, tap_off (per lane
// and half tile: where this tap of the lane's pixel lies in xt, or out of range for a tap in the padding) is not.
// HT: half tiles (of 32 pixels) per wave, 1 or 2.
template <int HT>
struct TapCursor {
    int step, cb, kw, kh;
    uint32_t tap;          // offset of tap (kh, kw) from a pixel's origin
    uint32_t cboff;        // offset of channel block cb from the tap
    uint32_t tap_off[2];

    __device__ __forceinline__ void place(const SharedParams& p, const bool (&live)[2], const int (&iy0)[2],
                                          const int (&ix0)[2], const uint32_t (&origin)[2])
    {
#pragma unroll
        for (int h = 0; h < HT; ++h) {
            const int iy = iy0[h] + kh, ix = ix0[h] + kw;
            const bool ok = live[h] && (unsigned)iy < (unsigned)p.tH && (unsigned)ix < (unsigned)p.tW;
            tap_off[h] = ok ? origin[h] + tap : kOutOfRange;
        }
    }
    // start at reduction step s (CB channel blocks per tap; cb_stride / row_stride: bytes between the channel blocks
    // of a pixel / the rows of an image)
    __device__ __forceinline__ void start(const SharedParams& p, int s, int CB, uint32_t cb_stride, uint32_t row_stride,
                                          const bool (&live)[2], const int (&iy0)[2], const int (&ix0)[2],
                                          const uint32_t (&origin)[2])
    {
        step = s;
        cb = kw = kh = 0;
        if (s != 0) {                                  // uniform; most calls start at the first step
            cb = s % CB;
            kw = (s / CB) % p.tKW;
            kh = (s / CB) / p.tKW;
        }
        tap = (uint32_t)kh * row_stride + (uint32_t)kw * 32u;
        cboff = (uint32_t)cb * cb_stride;
        place(p, live, iy0, ix0, origin);
    }
    // one step on; past the last step it stays where it is (that step is then simply requested again)
    __device__ __forceinline__ void advance(const SharedParams& p, int n_steps, int CB, uint32_t cb_stride,
                                            uint32_t row_stride, const bool (&live)[2], const int (&iy0)[2],
                                            const int (&ix0)[2], const uint32_t (&origin)[2])
    {
        if (step + 1 >= n_steps) return;
        ++step;
        cboff += cb_stride;
        if (++cb == CB) {
            cb = 0;
            cboff = 0;
            tap += 32u;
            if (++kw == p.tKW) { kw = 0; ++kh; tap += row_stride - (uint32_t)p.tKW * 32u; }
            place(p, live, iy0, ix0, origin);
        }
    }
};

// The two pixels of a lane (one per half tile of 32 pixels): image, output position, sample count, whether it takes
// part, the input position of tap (0, 0) and origin = offset in xt of xt[n][iy0][0][ix0][16 g] modulo 2^32 (only used
// with an in-image tap added).  Offsets into xt are 32 bits wide (the host keeps the buffer below 2 GB), so that an
// operand address is the uniform buffer plus one vector register.
template <int HT>
__device__ __forceinline__ void decode_half_tiles(const SharedParams& p, int64_t pix0, int col, int g, int CB, int64_t npix,
                                                  bool (&live)[2], int (&n_)[2], int (&oy_)[2], int (&ox_)[2],
                                                  int (&to_)[2], int (&iy0)[2], int (&ix0)[2], uint32_t (&origin)[2])
{
#pragma unroll
    for (int h = HT; h < 2; ++h) {                     // half tiles this wave does not have
        live[h] = false;
        n_[h] = oy_[h] = ox_[h] = to_[h] = iy0[h] = ix0[h] = 0;
        origin[h] = 0;
    }
#pragma unroll
    for (int h = 0; h < HT; ++h) {
        const int64_t pix = pix0 + 32 * h + col;
        const bool valid = pix < npix;
        const uint32_t pc = (uint32_t)(valid ? pix : npix - 1);       // the pixel count fits 32 bits (checked by the host)
        uint32_t ox, oy;
        const uint32_t row = div_mod(pc, (uint32_t)p.OW, p.inv_OW, ox);
        n_[h] = (int)div_mod(row, (uint32_t)p.OH, p.inv_OH, oy);
        ox_[h] = (int)ox;
        oy_[h] = (int)oy;
        live[h] = shared_pixel_range(p, pc, to_[h]) && valid;
        iy0[h] = oy_[h] * p.t_stride_h - p.t_pad_h;
        ix0[h] = ox_[h] * p.t_stride_w - p.t_pad_w;
        origin[h] = ((uint32_t)(n_[h] * p.tH + iy0[h]) * (uint32_t)(CB * p.tW) + (uint32_t)ix0[h]) * 32u + 16u * (uint32_t)g;
    }
}

// Values of the OUT template parameter (explained at the layer kernel).
enum { kOutPartial = 0, kOutAcc = 1, kOutRequant = 2 };

// The end of a wave's tile: what is done with the sums of its 32 channels x 64 pixels (see the OUT values below).
// acc[h][b]: digit plane b of half tile h; live / n_ / oy_ / ox_ / to_: this lane's pixel in each half tile.
template <int P, int OUT, int HT>
__device__ __forceinline__ void tile_epilogue(const SharedParams& p, v16i (&acc)[HT][P], const bool (&live)[2],
                                              const int (&n_)[2], const int (&oy_)[2], const int (&ox_)[2],
                                              const int (&to_)[2], int ocb, int lane, const float* s_mult,
                                              const float* s_bias)
{
    const int g = lane >> 5;
    // result row (channel) of register q: 8*(q/4) + 4*(lane/32) + q%4; column (pixel) = lane%32
    const int64_t plane = (int64_t)p.OH * p.OW;
    auto sum_of = [&](int h, int q) {                  // the digit planes recombined
        uint32_t u = 0;
#pragma unroll
        for (int b = 0; b < P; ++b) u += (uint32_t)acc[h][b][q] << (8 * b);
        return u;
    };
    // Per half tile, `full` (the block has 32 real channels) is a compile-time constant in the code below.
    auto finish = [&](auto full_c) {
        constexpr bool FULL = decltype(full_c)::value;
#pragma unroll
        for (int h = 0; h < HT; ++h) {
            if (!live[h]) continue;                    // uniform over a quad of lanes where that matters
            const int oc_first = ocb * 32 + 4 * g;     // channel of register 0; register q: + 8 (q / 4) + q % 4
            const int64_t o_first = ((int64_t)n_[h] * p.OC + oc_first) * plane + oy_[h] * p.OW + ox_[h];
            if constexpr (OUT == kOutPartial) {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int dq = 8 * (q >> 2) + (q & 3);
                    if (FULL || oc_first + dq < p.OC)   // exact in any order: the arithmetic is modulo 2^32
                        atomicAdd(&p.acc[o_first + dq * plane], (int32_t)sum_of(h, q));
                }
                continue;
            }
            const float inv_s = (to_[h] > 0) ? __fdiv_rn(1.0f, (float)to_[h]) : 0.0f;
            const bool has_bias = p.bias != nullptr;
            auto rescaled = [&](int q, uint32_t u) {    // the arithmetic of rescale()
                const int ocl = 8 * (q >> 2) + 4 * g + (q & 3);
                float r = __fmul_rn(__fmul_rn(__int2float_rn((int32_t)u), s_mult[ocl]), inv_s);
                if (has_bias) r = __fadd_rn(r, s_bias[ocl]);
                return r;
            };
            if constexpr (OUT == kOutAcc) {
                const bool with_y = p.y != nullptr;
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int dq = 8 * (q >> 2) + (q & 3);
                    if (!FULL && oc_first + dq >= p.OC) continue;
                    const uint32_t u = sum_of(h, q);
                    if (p.acc) p.acc[o_first + dq * plane] = (int32_t)u;
                    if (with_y) p.y[o_first + dq * plane] = rescaled(q, u);
                }
                continue;
            }
            // Requantised activations.  Every global operand (the residual) is loaded before the first store: a
            // store may alias a later load as far as the compiler can tell, and interleaving them would put the
            // latency of each load in series.
            const int j = lane & 3;
            // [N][OC][OH][OW] as words: lane j of a quad moves the word of channel (first of the group of four) + j,
            // pixels (pin & ~3) .. + 3, and the four lanes - consecutive pixels of one image - swap bytes
            const int64_t w_first = o_first + j * plane - ((oy_[h] * p.OW + ox_[h]) & 3);
            // blocked layout: the four channels of a register group are four consecutive bytes of the pixel's block
            const int64_t b_first = (((((int64_t)n_[h] * p.OH + oy_[h]) * gridDim.y + ocb) * p.OW + ox_[h]) << 5) + 4 * g;
            float res[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) res[q] = 0.0f;
            if (p.rq.res_f32) {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int dq = 8 * (q >> 2) + (q & 3);
                    if (FULL || oc_first + dq < p.OC) res[q] = p.rq.res_f32[o_first + dq * plane];
                }
            } else if (p.rq.res_i8 && (p.rq.res_blocked || p.quad_res)) {
                uint32_t resw[4];
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    resw[qq] = 0;
                    if (p.rq.res_blocked)
                        resw[qq] = *reinterpret_cast<const uint32_t*>(p.rq.res_i8 + b_first + 8 * qq);
                    else if (FULL || oc_first + 8 * qq + j < p.OC)
                        resw[qq] = *reinterpret_cast<const uint32_t*>(p.rq.res_i8 + w_first + 8 * qq * plane);
                }
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    // byte i: channel (first of the group) + i at this lane's pixel
                    const uint32_t w = p.rq.res_blocked ? resw[qq] : quad_transpose_bytes(resw[qq]);
#pragma unroll
                    for (int i = 0; i < 4; ++i) res[4 * qq + i] = __fmul_rn((float)(int8_t)(w >> (8 * i)), p.rq.res_step);
                }
            } else if (p.rq.res_i8) {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int dq = 8 * (q >> 2) + (q & 3);
                    if (FULL || oc_first + dq < p.OC)
                        res[q] = __fmul_rn((float)p.rq.res_i8[o_first + dq * plane], p.rq.res_step);
                }
            }
            const bool relu = p.rq.relu != 0;
            if (p.acc || p.y) {                        // rarely: the other outputs as well, in a pass of their own
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int dq = 8 * (q >> 2) + (q & 3);
                    if (!FULL && oc_first + dq >= p.OC) continue;
                    const uint32_t u = sum_of(h, q);
                    if (p.acc) p.acc[o_first + dq * plane] = (int32_t)u;
                    if (p.y) p.y[o_first + dq * plane] = rescaled(q, u);
                }
            }
            // The integers of requantize_one() with fewer instructions (32 outputs per lane make this loop a third
            // of a short layer's time): the bias and the residual are added unconditionally (they are 0.0 when
            // absent; that can only turn a -0.0 into +0.0, which rounds to the same integer), the ReLU gate and
            // the clamp are max/min (a NaN ends at lo either way, as inv_step is not negative - checked by the
            // host), and the conversion adds 1.5 * 2^23, which leaves the two's-complement byte in the low bits.
            const float floor_t = relu ? 0.0f : -__builtin_huge_valf();
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                uint32_t w[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int q = 4 * qq + i;
                    const int ocl = 8 * qq + 4 * g + i;
                    float t = __fmul_rn(__fmul_rn(__int2float_rn((int32_t)sum_of(h, q)), s_mult[ocl]), inv_s);
                    t = __fadd_rn(__fadd_rn(t, s_bias[ocl]), res[q]);
                    t = __builtin_fmaxf(t, floor_t);
                    float v = rintf(__fmul_rn(t, p.rq.inv_step));
                    v = __builtin_fminf(__builtin_fmaxf(v, p.rq.lo), p.rq.hi);
                    w[i] = __float_as_uint(__fadd_rn(v, 12582912.0f));
                    if (!FULL && oc_first + 8 * qq + i >= p.OC) w[i] = 0;   // padding channels of the blocked layout
                }
                // byte 0 of w[0..3] -> bytes 0..3
                uint32_t word = __builtin_amdgcn_perm(w[1], w[0], 0x0c0c0400u) | __builtin_amdgcn_perm(w[3], w[2], 0x04000c0cu);
                if (p.rq.out_blocked) {
                    *reinterpret_cast<uint32_t*>(p.rq.x_out + b_first + 8 * qq) = word;
                } else if (p.quad_store) {
                    word = quad_transpose_bytes(word); // byte i: this lane's channel at pixel (pin & ~3) + i
                    if (FULL || oc_first + 8 * qq + j < p.OC)
                        *reinterpret_cast<uint32_t*>(p.rq.x_out + w_first + 8 * qq * plane) = word;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (FULL || oc_first + 8 * qq + i < p.OC)
                            p.rq.x_out[o_first + (8 * qq + i) * plane] = (int8_t)(word >> (8 * i));
                }
            }
        }
    };
    if (ocb * 32 + 32 <= p.OC) finish(std::true_type{});
    else finish(std::false_type{});
}

// What a workgroup does with its sums: add them to the accumulators atomically (masked or split reductions; the
// rescaling is a separate pass then), store accumulators (and rescaled values), or store requantised activations
// (and, if asked for, the other two).  A template parameter, so that the unrolled epilogue is straight-line code.

// Two waves per SIMD must stay resident (512 registers per lane and SIMD, accumulators included): left alone the
// compiler takes 162 + 96 for the requantising two-half-tile variant, and a layer with more than 256 workgroups
// then needs a second round.  (Four planes and two half tiles, 128 accumulators, do not fit twice without spills.)
template <int P, int OUT, int HT>
__global__ void __launch_bounds__(256, (P == 4 && HT == 2) ? 1 : 2) k_conv_shared_mfma(const SharedParams p)
{
    __shared__ v4i a_lds[kStageSteps * P * 64];
    __shared__ float s_mult[32], s_bias[32];       // rescale factors of this block of channels (read after the loop)
    __shared__ int s_takes_part[4];                // per wave: one of its pixels takes part in the segment voted on

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    // Workgroups are dealt to the 8 XCDs round-robin by their index; each XCD has its own L2.  Renumber them so
    // that every XCD works on one contiguous eighth of the pixel tiles (lengths differing by at most one tile) and
    // its L2 only has to hold that part of the input.  (The launcher rounds the grid up to a multiple of 8.)
    const unsigned n_tiles = (unsigned)((npix + 128 * HT - 1) / (128 * HT));
    const unsigned wg = xcd_contiguous(blockIdx.x, n_tiles);
    if (wg == 0xFFFFFFFFu) return;                 // uniform over the workgroup, before any barrier
    const int64_t pix0 = ((int64_t)wg * 4 + wave) * (32 * HT);
    const int ocb = blockIdx.y;

    const int CB = p.C_pad >> 5;
    const int n_steps = p.tKH * p.tKW * CB;
    // this workgroup's part of the reduction
    const int per_split = (n_steps + p.ksplit - 1) / p.ksplit;
    const int s_begin = (int)blockIdx.z * per_split;
    const int s_end = min(n_steps, s_begin + per_split);
    const int8_t* const wblock0 = p.planes + (int64_t)ocb * p.n_ksteps * (kMaxPlanes * kPlaneStride);
    const int8_t* wblock = wblock0;                // the channel block in the planes of the current segment

    // weights: operand i of a chunk (i = (step * P + plane) * 64 + lane) is fetched by thread i mod 256; its byte
    // offset inside the chunk is fixed.  A chunk may reach past the last step: the buffer is padded by one chunk
    // (those operands are staged but never multiplied).
    constexpr int kStageRegs = kStageSteps * P * 64 / 256;
    v4i stage[kStageRegs];
    uint32_t woff[kStageRegs];
#pragma unroll
    for (int r = 0; r < kStageRegs; ++r) {
        const int i = r * 256 + (int)threadIdx.x;
        woff[r] = (uint32_t)((((i / (P * 64)) * kMaxPlanes + (i >> 6) % P) * 64 + (i & 63)) * 16);
    }
    // Buffer loads: the address of an operand is the (uniform) block of this channel block and segment, a scalar
    // offset for the chunk and the thread's fixed offset - no per-load address arithmetic in vector registers, which
    // the compiler would otherwise do in registers it also uses for operands, making every first LDS read of a chunk
    // wait for the weight loads that were just issued.
    __amdgpu_buffer_rsrc_t w_rsrc = operand_buffer(wblock, (uint32_t)(p.n_ksteps + kStageSteps) * (kMaxPlanes * kPlaneStride));
    auto fetch_weights = [&](int s0) {
        const uint32_t chunk = (uint32_t)s0 * (uint32_t)(kMaxPlanes * kPlaneStride);   // uniform
#pragma unroll
        for (int r = 0; r < kStageRegs; ++r) stage[r] = load_operand(w_rsrc, woff[r], chunk);
    };

    fetch_weights(s_begin);          // first of all: nothing below depends on it until the first barrier

    bool live[2];
    int n_[2], oy_[2], ox_[2], to_[2], iy0[2], ix0[2];
    uint32_t origin[2];
    decode_half_tiles<HT>(p, pix0, col, g, CB, npix, live, n_, oy_, ox_, to_, iy0, ix0, origin);
    // a wave without any pixel that takes part still helps to stage the weights (and keeps the barriers whole)
    const bool active = __ballot(live[0] || live[1]) != 0ull;

    v16i acc[HT][P];
#pragma unroll
    for (int h = 0; h < HT; ++h)
#pragma unroll
        for (int b = 0; b < P; ++b)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[h][b][q] = 0;

    const uint32_t cb_stride = (uint32_t)p.tW * 32u;            // bytes between the channel blocks of one pixel
    const uint32_t row_stride = (uint32_t)CB * cb_stride;       // ... between the rows of one image
    const __amdgpu_buffer_rsrc_t xt_rsrc = operand_buffer(p.xt, p.xt_bytes);
    if (OUT != kOutPartial && threadIdx.x < 32) {    // visible to every wave after the loop's first barrier
        const int oc = ocb * 32 + (int)threadIdx.x;
        s_mult[threadIdx.x] = (p.mult && oc < p.OC) ? p.mult[oc] : p.default_mult;
        s_bias[threadIdx.x] = (p.bias && oc < p.OC) ? p.bias[oc] : 0.0f;
    }

    // One pass over the reduction per segment of the sample axis (one pass when there are no segments).  The passes
    // accumulate into the same registers: a pixel that does not take part in a segment feeds zeros, because its
    // operand offsets are out of range.
    const int n_seg = p.n_seg > 0 ? p.n_seg : 1;
    for (int seg = 0; seg < n_seg; ++seg) {
        bool lv[2] = {live[0], live[1]};             // pixels that take part in this pass
        if (p.n_seg > 0) {
#pragma unroll
            for (int h = 0; h < 2; ++h) lv[h] = live[h] && to_[h] >= p.seg_level[seg];
            if (seg > 0) {
                // Levels nest: when no pixel of the workgroup reaches this one, none reaches a later one.  The
                // decision has to be the workgroup's (the passes have barriers).  The votes of two segments cannot
                // mix: a pass, with its barriers, lies between them.
                const int mine = (__ballot(lv[0] || lv[1]) != 0ull) ? 1 : 0;       // taken by the whole wave
                if (lane == 0) s_takes_part[wave] = mine;
                __syncthreads();
                if ((s_takes_part[0] | s_takes_part[1] | s_takes_part[2] | s_takes_part[3]) == 0) break;
                wblock = wblock0 + (int64_t)seg * p.seg_stride;
                w_rsrc = operand_buffer(wblock, (uint32_t)(p.n_ksteps + kStageSteps) * (kMaxPlanes * kPlaneStride));
                fetch_weights(s_begin);
            }
        }
        const bool active_seg = __ballot(lv[0] || lv[1]) != 0ull;
        TapCursor<HT> cur;
        cur.start(p, min(s_begin, n_steps - 1), CB, cb_stride, row_stride, lv, iy0, ix0, origin);
        // one-half-tile waves run alone or nearly alone on their SIMD (that is when they are chosen) and have registers
        // to spare: a deeper pipeline hides more of the load latency there (stage 4 of ResNet-18: 28 -> 24.5 us)
        constexpr int kDepthT = HT == 1 ? kStageSteps : kDepth;
        v4i opb[kDepthT][HT];
        auto request = [&](int slot) {
#pragma unroll
            for (int h = 0; h < HT; ++h) opb[slot][h] = load_operand(xt_rsrc, cur.tap_off[h], cur.cboff);
            cur.advance(p, n_steps, CB, cb_stride, row_stride, lv, iy0, ix0, origin);
        };

        if (active_seg) {
#pragma unroll
            for (int d = 0; d < kDepthT; ++d) request(d);
        }
        for (int s0 = s_begin; s0 < s_end; s0 += kStageSteps) {
            __syncthreads();                             // the previous chunk has been consumed by every wave
#pragma unroll
            for (int r = 0; r < kStageRegs; ++r) a_lds[r * 256 + threadIdx.x] = stage[r];
            __syncthreads();
            // unconditional, like the activation requests (past the last chunk it reads the padding chunk of the
            // buffer, or the next block's first chunk): a branch around it makes the compiler's wait counts assume
            // the path without loads, and the first LDS reads of every chunk then wait for loads just issued
            fetch_weights(s0 + kStageSteps);
            if (active_seg) {
                // the weight operands of step ks + 1 are read from LDS while the matrix instructions of step ks run
                v4i a[2][P];
#pragma unroll
                for (int b = 0; b < P; ++b) a[0][b] = a_lds[b * 64 + lane];
#pragma unroll
                for (int ks = 0; ks < kStageSteps; ++ks) {
                    const int d = ks % kDepthT;
                    if (ks + 1 < kStageSteps) {
#pragma unroll
                        for (int b = 0; b < P; ++b) a[(ks + 1) & 1][b] = a_lds[((ks + 1) * P + b) * 64 + lane];
                    }
                    if (s0 + ks < s_end) {               // wave-uniform
#pragma unroll
                        for (int b = 0; b < P; ++b)
#pragma unroll
                            for (int h = 0; h < HT; ++h)
                                acc[h][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[ks & 1][b], opb[d][h], acc[h][b], 0, 0, 0);
                    }
                    request(d);     // unconditional (past the end: the last step again), so that the number of
                                    // loads in flight is the same on every path and no wait is longer than needed
                }
            }
        }
    }
    if (!active) return;

    tile_epilogue<P, OUT, HT>(p, acc, live, n_, oy_, ox_, to_, ocb, lane, s_mult, s_bias);
}

// Short reductions (all weight operands of a channel block fit LDS: the first layer of a network, 3x3 layers on 64
// channels, 1x1 shortcuts, classifiers): a persistent variant.  A workgroup stages the whole block once and then walks
// over pixel tiles, `columns` apart; inside the walk there is no barrier and no staging, the kernel arguments and
// the rescale factors are read once, and the four waves run independently of each other.  Unsplit, unmasked calls
// only.  Dynamic LDS: n_steps * P * 1024 bytes.  gridDim.x is a multiple of 8, columns = the grid the plain kernel
// would get.  HT: half tiles of 32 pixels per wave (a tile of the walk is 128 HT pixels).
template <int P, int OUT, int HT>
__global__ void __launch_bounds__(256, HT == 1 ? 4 : 2) k_conv_shared_mfma_resident(const SharedParams p, unsigned columns)
{
    extern __shared__ v4i a_all[];                 // [n_steps][P][64]
    __shared__ float s_mult[32], s_bias[32];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    const int ocb = blockIdx.y;
    const int CB = p.C_pad >> 5;
    const int n_steps = p.tKH * p.tKW * CB;
    const int8_t* wblock = p.planes + (int64_t)ocb * p.n_ksteps * (kMaxPlanes * kPlaneStride);
    for (int i = threadIdx.x; i < n_steps * P * 64; i += 256) {
        const int step = i / (P * 64), b = (i >> 6) % P;
        a_all[i] = *reinterpret_cast<const v4i*>(wblock + ((int64_t)(step * kMaxPlanes + b) * 64 + (i & 63)) * 16);
    }
    if (threadIdx.x < 32) {
        const int oc = ocb * 32 + (int)threadIdx.x;
        s_mult[threadIdx.x] = (p.mult && oc < p.OC) ? p.mult[oc] : p.default_mult;
        s_bias[threadIdx.x] = (p.bias && oc < p.OC) ? p.bias[oc] : 0.0f;
    }
    __syncthreads();

    const uint32_t cb_stride = (uint32_t)p.tW * 32u;
    const uint32_t row_stride = (uint32_t)CB * cb_stride;
    const __amdgpu_buffer_rsrc_t xt_rsrc = operand_buffer(p.xt, p.xt_bytes);
    const unsigned n_tiles = (unsigned)((npix + 128 * HT - 1) / (128 * HT));
    for (unsigned v = blockIdx.x; v < columns; v += gridDim.x) {
        const unsigned wg = xcd_contiguous(v, n_tiles);     // each XCD keeps one contiguous eighth of the pixel tiles
        if (wg == 0xFFFFFFFFu) continue;
        const int64_t pix0 = ((int64_t)wg * 4 + wave) * (32 * HT);
        bool live[2];
        int n_[2], oy_[2], ox_[2], to_[2], iy0[2], ix0[2];
        uint32_t origin[2];
        decode_half_tiles<HT>(p, pix0, col, g, CB, npix, live, n_, oy_, ox_, to_, iy0, ix0, origin);
        if (__ballot(live[0] || live[1]) == 0ull) continue;      // wave-uniform; no barrier below

        v16i acc[HT][P];
#pragma unroll
        for (int h = 0; h < HT; ++h)
#pragma unroll
            for (int b = 0; b < P; ++b)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[h][b][q] = 0;

        TapCursor<HT> cur;
        cur.start(p, 0, CB, cb_stride, row_stride, live, iy0, ix0, origin);
        v4i opb[kDepth][HT];
        auto request = [&](int slot) {
#pragma unroll
            for (int h = 0; h < HT; ++h) opb[slot][h] = load_operand(xt_rsrc, cur.tap_off[h], cur.cboff);
            cur.advance(p, n_steps, CB, cb_stride, row_stride, live, iy0, ix0, origin);
        };
#pragma unroll
        for (int d = 0; d < kDepth; ++d) request(d);

        v4i a[2][P];
#pragma unroll
        for (int b = 0; b < P; ++b) a[0][b] = a_all[b * 64 + lane];
        for (int s0 = 0; s0 < n_steps; s0 += kDepth) {
#pragma unroll
            for (int ks = 0; ks < kDepth; ++ks) {
                const int nxt = min(s0 + ks + 1, n_steps - 1);       // the operands of the next step, one step ahead
#pragma unroll
                for (int b = 0; b < P; ++b) a[(ks + 1) & 1][b] = a_all[(nxt * P + b) * 64 + lane];
                if (s0 + ks < n_steps) {             // wave-uniform
#pragma unroll
                    for (int b = 0; b < P; ++b)
#pragma unroll
                        for (int h = 0; h < HT; ++h)
                            acc[h][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[ks & 1][b], opb[ks][h], acc[h][b], 0, 0, 0);
                }
                request(ks);
            }
        }
        tile_epilogue<P, OUT, HT>(p, acc, live, n_, oy_, ox_, to_, ocb, lane, s_mult, s_bias);
    }
}

// 3 x 3 layers with unit stride and one pixel of padding on the blocked layout: BOTH operands come from LDS.
// The plain kernel fetches each activation operand straight from global memory, once per tap: two 16-byte loads per
// lane and reduction step, which the path from L2 through L1 into the registers of eight waves cannot deliver as fast
// as the matrix cores consume them.  Here the reduction runs channel block by channel block; for the current block of
// 32 input channels a team of four waves keeps, next to the nine taps' weight operands, the WINDOW of the input
// that its pixel tile touches: all positions from the first pixel's tap (0, 0) to the last pixel's tap (2, 2), in a
// "virtual" row-major order in which every image row is preceded by one zero position (its left padding, and the
// right padding of the row before) and every image by one zero row.  In that order tap (kh, kw) of output pixel
// (n, oy, ox) is at  ((n (H + 1) + oy + kh) (W + 1) + ox + kw)  - the pixel's own position plus a uniform offset - so
// an activation operand is one 16-byte LDS read at  (lane's slot + kh (W + 1) + kw)  and the nine taps of a pixel
// re-use what was fetched once.  The two 16-channel halves of a position live in two half planes, so that the lanes
// of a half tile read consecutive 16-byte words.
//
// TEAMS > 1: few pixel tiles and a long reduction - the channel blocks are dealt to TEAMS teams of four waves that
// work on the SAME pixels with their own LDS regions; their sums meet in LDS at the end and team 0 runs the
// epilogue.  This gives every SIMD two waves to interleave where the tile count alone would give it one.
//
// Unsplit calls (p.ksplit = 1); pixels that do not take part in the call feed zeros and are not stored.
// WS: window slots / 256.  Dynamic LDS: TEAMS * (kAregs + 2 WS) * 4096 bytes.
template <int P, int OUT, int HT, int TEAMS, int WS>
__global__ void __launch_bounds__(256 * TEAMS, 2) k_conv3x3_window(const SharedParams p)
{
    extern __shared__ v4i win_lds[];
    __shared__ float s_mult[32], s_bias[32];
    __shared__ int s_segments;                     // segments of the sample axis that some pixel of the workgroup reaches
    constexpr int kTaps = 9;
    constexpr int kAregs = (kTaps * P * 64 + 255) / 256;        // 16-byte weight words per thread and channel block
    constexpr int kTeamWords = (kAregs + 2 * WS) * 256;         // v4i per team

    const int team = (int)threadIdx.x >> 8, tid = (int)threadIdx.x & 255;
    const int lane = threadIdx.x & 63, wave = ((int)threadIdx.x >> 6) & 3;
    const int col = lane & 31, g = lane >> 5;
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    constexpr int kTile = 128 * HT;                             // pixels of a workgroup
    const unsigned n_tiles = (unsigned)((npix + kTile - 1) / kTile);
    unsigned wg;
    int ocb;
    if (p.xcd_by_channels) {
        // the grid is n_tiles x (a multiple of 8 channel blocks); workgroup L of the launch runs on XCD L mod 8, which
        // owns gridDim.y / 8 consecutive channel blocks: its L2 holds their weights and the (small) input
        const unsigned linear = blockIdx.y * gridDim.x + blockIdx.x, local = linear >> 3, per_xcd = gridDim.y >> 3;
        ocb = (int)((linear & 7u) * per_xcd + local % per_xcd);
        wg = local / per_xcd;
    } else {
        wg = xcd_contiguous(blockIdx.x, n_tiles);
        if (wg == 0xFFFFFFFFu) return;             // uniform over the workgroup, before any barrier
        ocb = blockIdx.y;
    }
    const int64_t pix_first = (int64_t)wg * kTile;
    const int64_t pix0 = pix_first + wave * (32 * HT);
    const int CB = p.C_pad >> 5;
    const int cb_per_team = CB / TEAMS;            // the host checks that it divides
    const int cb_begin = team * cb_per_team;
    v4i* const a_lds = win_lds + team * kTeamWords;             // [tap][plane][lane]
    v4i* const b_lds = a_lds + kAregs * 256;                    // [half][slot]

    // weights: word i = (tap * P + plane) * 64 + lane of a channel block's chunk is fetched by thread i mod 256
    const int8_t* const wblock = p.planes + (int64_t)ocb * p.n_ksteps * (kMaxPlanes * kPlaneStride);
    auto segment_planes = [&](int seg) {           // the channel block in the digit planes of a segment's filter
        return operand_buffer(wblock + (int64_t)seg * (int64_t)p.seg_stride, (uint32_t)(p.n_ksteps + kStageSteps) * (kMaxPlanes * kPlaneStride));
    };
    __amdgpu_buffer_rsrc_t w_rsrc = segment_planes(0);
    v4i stage_a[kAregs];
    uint32_t woff[kAregs];
#pragma unroll
    for (int r = 0; r < kAregs; ++r) {
        const int i = r * 256 + tid;
        const int t = i / (P * 64), b = (i >> 6) % P;
        // reduction step of (tap t, channel block cb) = t * CB + cb; words past the ninth tap read as zeros
        woff[r] = t < kTaps ? (uint32_t)((((t * CB) * kMaxPlanes + b) * 64 + (i & 63)) * 16) : kOutOfRange;
    }
    auto fetch_weights = [&](int cb) {
        const uint32_t chunk = (uint32_t)cb * (uint32_t)(kMaxPlanes * kPlaneStride);      // uniform
#pragma unroll
        for (int r = 0; r < kAregs; ++r) stage_a[r] = load_operand(w_rsrc, woff[r], chunk);
    };
    fetch_weights(cb_begin);         // first of all: nothing below depends on it until the first barrier

    // the window: slot s holds virtual position q_first + s
    const int W1 = p.tW + 1, H1 = p.tH + 1;
    auto virtual_position = [&](uint32_t pix) {
        uint32_t ox, oy;
        const uint32_t row = div_mod(pix, (uint32_t)p.OW, p.inv_OW, ox);
        const uint32_t n = div_mod(row, (uint32_t)p.OH, p.inv_OH, oy);
        return (n * (uint32_t)H1 + oy) * (uint32_t)W1 + ox;
    };
    const uint32_t pix_last = (uint32_t)(min(pix_first + kTile, npix) - 1);
    const uint32_t q_first = virtual_position((uint32_t)pix_first);
    const uint32_t n_slots = virtual_position(pix_last) - q_first + 2u * (uint32_t)W1 + 3u;   // at most 256 WS (host)
    const uint32_t cb_stride = (uint32_t)p.tW * 32u;            // bytes between the channel blocks of one pixel
    const __amdgpu_buffer_rsrc_t xt_rsrc = operand_buffer(p.xt, p.xt_bytes);
    v4i stage_b[WS][2];
    uint32_t goff[WS];               // slot e * 256 + tid: offset of its position in channel block 0, or out of range
#pragma unroll
    for (int e = 0; e < WS; ++e) {
        const uint32_t s = (uint32_t)(e * 256 + tid);
        const uint32_t q = q_first + s;
        uint32_t vc, rr;
        const uint32_t vr = div_mod(q, (uint32_t)W1, p.inv_W1, vc);
        const uint32_t n = div_mod(vr, (uint32_t)H1, p.inv_H1, rr);
        const bool ok = s < n_slots && vc >= 1u && rr >= 1u && n < (uint32_t)p.N;
        goff[e] = ok ? (((n * (uint32_t)p.tH + (rr - 1u)) * (uint32_t)CB) * (uint32_t)p.tW + (vc - 1u)) * 32u : kOutOfRange;
    }
    auto fetch_window = [&](int cb) {
        const uint32_t block = (uint32_t)cb * cb_stride;                                    // uniform
#pragma unroll
        for (int e = 0; e < WS; ++e) {
            stage_b[e][0] = load_operand(xt_rsrc, goff[e], block);
            stage_b[e][1] = load_operand(xt_rsrc, goff[e] + 16u, block);     // out of range stays out of range
        }
    };
    fetch_window(cb_begin);

    bool live[2];
    int n_[2], oy_[2], ox_[2], to_[2], iy0[2], ix0[2];
    uint32_t origin[2];
    decode_half_tiles<HT>(p, pix0, col, g, CB, npix, live, n_, oy_, ox_, to_, iy0, ix0, origin);
    const bool active = __ballot(live[0] || live[1]) != 0ull;
    // this lane's operand of tap (kh, kw) and half tile h: b_lds[row_slot[h][kh] + kw]
    int row_slot[HT][3];
#pragma unroll
    for (int h = 0; h < HT; ++h) {
        const int slot = (int)(((uint32_t)(n_[h] * H1 + oy_[h])) * (uint32_t)W1 + (uint32_t)ox_[h] - q_first);
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) row_slot[h][kh] = g * (WS * 256) + slot + kh * W1;
    }

    v16i acc[HT][P];
#pragma unroll
    for (int h = 0; h < HT; ++h)
#pragma unroll
        for (int b = 0; b < P; ++b)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[h][b][q] = 0;

    if (OUT != kOutPartial && threadIdx.x < 32) {    // visible to every wave after the loop's first barrier
        const int oc = ocb * 32 + (int)threadIdx.x;
        s_mult[threadIdx.x] = (p.mult && oc < p.OC) ? p.mult[oc] : p.default_mult;
        s_bias[threadIdx.x] = (p.bias && oc < p.OC) ? p.bias[oc] : 0.0f;
    }

    // Budget map with announced levels (p.n_seg > 0): one pass over the channel blocks per segment of the sample axis,
    // each with its own filter, into the same sums; a pixel that does not reach a segment feeds zeros.  Levels nest,
    // so the workgroup runs the first n_seg segments, n_seg = the most that any of its pixels reaches.
    int n_seg = 1;
    if (p.n_seg > 0) {
        int reached = 0;                             // wave-uniform
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i < p.n_seg && __ballot((live[0] && to_[0] >= p.seg_level[i]) || (live[1] && to_[1] >= p.seg_level[i])) != 0ull)
                reached = i + 1;
        if (threadIdx.x == 0) s_segments = 0;
        __syncthreads();
        if (lane == 0 && reached > 0) atomicMax(&s_segments, reached);
        __syncthreads();
        n_seg = max(s_segments, 1);                  // (a pass over nothing but zeros when no pixel takes part at all)
    }
    int seg = 0, c = 0;
    for (int it = 0; it < n_seg * cb_per_team; ++it) {
        __syncthreads();                             // the previous channel block has been consumed by every wave
#pragma unroll
        for (int r = 0; r < kAregs; ++r) a_lds[r * 256 + tid] = stage_a[r];
#pragma unroll
        for (int e = 0; e < WS; ++e) {
            b_lds[e * 256 + tid] = stage_b[e][0];
            b_lds[WS * 256 + e * 256 + tid] = stage_b[e][1];
        }
        __syncthreads();
        // the next block's operands travel while this one is multiplied (after the last block: the same again, so
        // that the loads in flight are the same on every path)
        bool lv[2] = {live[0], live[1]};             // pixels that take part in this segment
        if (p.n_seg > 0) {
#pragma unroll
            for (int h = 0; h < 2; ++h) lv[h] = live[h] && to_[h] >= p.seg_level[seg];
        }
        int c_next = c + 1, seg_next = seg;
        if (c_next == cb_per_team && seg + 1 < n_seg) { c_next = 0; seg_next = seg + 1; w_rsrc = segment_planes(seg_next); }
        c_next = min(c_next, cb_per_team - 1);
        fetch_weights(cb_begin + c_next);
        fetch_window(cb_begin + c_next);
        c = c_next;
        seg = seg_next;

        v4i a[2][P], b[2][HT];
        auto activation = [&](int h, int at) {       // zeros for a pixel outside the segment
            const v4i v = b_lds[at];
            return lv[h] ? v : v4i{0, 0, 0, 0};
        };
#pragma unroll
        for (int pl = 0; pl < P; ++pl) a[0][pl] = a_lds[pl * 64 + lane];
#pragma unroll
        for (int h = 0; h < HT; ++h) b[0][h] = activation(h, row_slot[h][0]);
#pragma unroll
        for (int t = 0; t < kTaps; ++t) {
            if (t + 1 < kTaps) {
                const int kh = (t + 1) / 3, kw = (t + 1) % 3;
#pragma unroll
                for (int pl = 0; pl < P; ++pl) a[(t + 1) & 1][pl] = a_lds[((t + 1) * P + pl) * 64 + lane];
#pragma unroll
                for (int h = 0; h < HT; ++h) b[(t + 1) & 1][h] = activation(h, row_slot[h][kh] + kw);
            }
#pragma unroll
            for (int pl = 0; pl < P; ++pl)
#pragma unroll
                for (int h = 0; h < HT; ++h)
                    acc[h][pl] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[t & 1][pl], b[t & 1][h], acc[h][pl], 0, 0, 0);
        }
    }

    if constexpr (TEAMS > 1) {
        // the teams' sums meet in LDS: team k > 0 leaves its registers at [k - 1][wave][register quad][lane]
        constexpr int kQuads = HT * P * 4;
        __syncthreads();                             // every operand has been read
        if (team > 0) {
            v4i* const dst = win_lds + (((team - 1) * 4 + wave) * kQuads) * 64 + lane;
#pragma unroll
            for (int h = 0; h < HT; ++h)
#pragma unroll
                for (int pl = 0; pl < P; ++pl)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4)
                        dst[((h * P + pl) * 4 + q4) * 64] = v4i{acc[h][pl][4 * q4], acc[h][pl][4 * q4 + 1], acc[h][pl][4 * q4 + 2], acc[h][pl][4 * q4 + 3]};
        }
        __syncthreads();
        if (team > 0) return;
#pragma unroll
        for (int k = 1; k < TEAMS; ++k) {
            const v4i* const src = win_lds + (((k - 1) * 4 + wave) * kQuads) * 64 + lane;
#pragma unroll
            for (int h = 0; h < HT; ++h)
#pragma unroll
                for (int pl = 0; pl < P; ++pl)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const v4i v = src[((h * P + pl) * 4 + q4) * 64];
                        acc[h][pl][4 * q4] += v.x; acc[h][pl][4 * q4 + 1] += v.y;
                        acc[h][pl][4 * q4 + 2] += v.z; acc[h][pl][4 * q4 + 3] += v.w;
                    }
        }
    }
    if (!active) return;

    tile_epilogue<P, OUT, HT>(p, acc, live, n_, oy_, ox_, to_, ocb, lane, s_mult, s_bias);
}

// Any layer shape: one output pixel per lane, one output channel per workgroup row.  (Grouping the taps' loads
// here, with (channel, kh, kw) stepped at run time, measured slower than this plain loop: the stepping is more
// scalar work per tap than the loop counters; 3 x 3 depthwise layers have the unrolled kernel below instead.)
__global__ void __launch_bounds__(256) k_conv_shared_direct(const SharedParams p)
{
    const int oc = blockIdx.y;
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    const int64_t pix = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pix >= npix) return;
    int to;
    if (!shared_pixel_range(p, pix, to)) return;
    const uint32_t pix32 = (uint32_t)pix;                  // the number of outputs fits 32 bits, so pixels do too
    const uint32_t row32 = pix32 / (uint32_t)p.OW;
    const int ox = (int)(pix32 - row32 * (uint32_t)p.OW);
    const int n = (int)(row32 / (uint32_t)p.OH);
    const int oy = (int)(row32 - (uint32_t)n * (uint32_t)p.OH);
    const int grp = oc / p.OCg;
    const int32_t* wrow = p.w32 + (int64_t)oc * p.K;
    // the activation tensor has fewer than 2^31 elements: 32-bit indices
    const uint32_t xn = (uint32_t)(n * p.C + grp * p.Cg) * (uint32_t)(p.H * p.W);
    const int iy0 = oy * p.stride_h - p.pad_h, ix0 = ox * p.stride_w - p.pad_w;
    uint32_t sum = 0;
    int k = 0;
    for (int ci = 0; ci < p.Cg; ++ci)
        for (int kh = 0; kh < p.KH; ++kh) {
            const int iy = iy0 + kh;
            const uint32_t row = xn + (uint32_t)(ci * p.H + iy) * (uint32_t)p.W;
            for (int kw = 0; kw < p.KW; ++kw, ++k) {
                const int ix = ix0 + kw;
                if ((unsigned)iy >= (unsigned)p.H || (unsigned)ix >= (unsigned)p.W) continue;
                sum += (uint32_t)((int32_t)p.x[row + (uint32_t)ix] * wrow[k]);   // modulo 2^32
            }
        }
    const int64_t o = (((int64_t)n * p.OC + oc) * p.OH + oy) * p.OW + ox;
    if (p.masked) {
        p.acc[o] = (int32_t)((uint32_t)p.acc[o] + sum);
    } else {
        if (p.acc) p.acc[o] = (int32_t)sum;
        emit(p, o, oc, (int32_t)sum, to);
    }
}

// Depthwise layers (one input channel per group) with a kernel size known at compile time: the taps' offsets and
// their inside-the-image tests do not depend on the channel, so a lane computes them once and then walks over
// `channels` output channels, two at a time, with every load of a pair requested before the first is used
// (range-checked buffer loads: a tap in the padding has an offset beyond the tensor and reads as zero).
template <int KH, int KW>
__global__ void __launch_bounds__(256) k_conv_shared_depthwise(const SharedParams p, int channels)
{
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    const int64_t pix = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pix >= npix) return;
    int to;
    if (!shared_pixel_range(p, pix, to)) return;
    const uint32_t pix32 = (uint32_t)pix;                  // the number of outputs fits 32 bits, so pixels do too
    const uint32_t row32 = pix32 / (uint32_t)p.OW;
    const int ox = (int)(pix32 - row32 * (uint32_t)p.OW);
    const int n = (int)(row32 / (uint32_t)p.OH);
    const int oy = (int)(row32 - (uint32_t)n * (uint32_t)p.OH);
    const __amdgpu_buffer_rsrc_t x_rsrc = operand_buffer(p.x, (uint32_t)((int64_t)p.N * p.C * p.H * p.W));
    const int iy0 = oy * p.stride_h - p.pad_h, ix0 = ox * p.stride_w - p.pad_w;
    constexpr int T = KH * KW;
    uint32_t rel[T];           // offset of the tap inside an image plane; beyond the tensor when outside the image
#pragma unroll
    for (int kh = 0; kh < KH; ++kh)
#pragma unroll
        for (int kw = 0; kw < KW; ++kw) {
            const int iy = iy0 + kh, ix = ix0 + kw;
            const bool ok = ((unsigned)iy < (unsigned)p.H) & ((unsigned)ix < (unsigned)p.W);
            rel[kh * KW + kw] = ok ? (uint32_t)(iy * p.W + ix) : kOutOfRange;
        }
    const uint32_t plane = (uint32_t)(p.H * p.W);
    const int oc_end = min(p.OC, ((int)blockIdx.y + 1) * channels);
    for (int oc0 = (int)blockIdx.y * channels; oc0 < oc_end; oc0 += 2) {
        const int oc1 = min(oc0 + 1, oc_end - 1);          // a single last channel is computed twice, stored once
        int32_t xa[T], xb[T];
        const uint32_t base_a = (uint32_t)(n * p.C + oc0 / p.OCg) * plane;     // plane starts are below 2^31, so
        const uint32_t base_b = (uint32_t)(n * p.C + oc1 / p.OCg) * plane;     // base + kOutOfRange stays beyond
#pragma unroll
        for (int u = 0; u < T; ++u) {
            xa[u] = (int32_t)(int8_t)__builtin_amdgcn_raw_buffer_load_b8(x_rsrc, (int)(base_a + rel[u]), 0, 0);
            xb[u] = (int32_t)(int8_t)__builtin_amdgcn_raw_buffer_load_b8(x_rsrc, (int)(base_b + rel[u]), 0, 0);
        }
        const int32_t* wa = p.w32 + (int64_t)oc0 * T;
        const int32_t* wb = p.w32 + (int64_t)oc1 * T;
        uint32_t sum_a = 0, sum_b = 0;
#pragma unroll
        for (int u = 0; u < T; ++u) {
            sum_a += (uint32_t)(xa[u] * wa[u]);            // modulo 2^32
            sum_b += (uint32_t)(xb[u] * wb[u]);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int oc = h ? oc1 : oc0;
            const uint32_t sum = h ? sum_b : sum_a;
            if (h && oc1 == oc0) break;
            const int64_t o = (((int64_t)n * p.OC + oc) * p.OH + oy) * p.OW + ox;
            if (p.masked) {
                p.acc[o] = (int32_t)((uint32_t)p.acc[o] + sum);
            } else {
                if (p.acc) p.acc[o] = (int32_t)sum;
                emit(p, o, oc, (int32_t)sum, to);
            }
        }
    }
}

// Digit planes needed for |W| <= m = 2 * n_samples * 2^max_shift.  P balanced digits represent every integer
// in [-128 R, 127 R], R = (256^P - 1) / 255, which contains [-2^(8P-2), 2^(8P-2)]: two bits above the
// length of m are enough (one would not be: 32640 = 255 * 128 has 15 bits and needs three digits).
// With four planes the last digit may wrap, which is exact modulo 2^32.
inline int planes_needed(int max_shift, int n_samples)
{
    int bits = 2;
    for (int64_t m = ((int64_t)2 * n_samples) << max_shift; m > 0; m >>= 1) bits++;
    const int planes = (bits + 7) / 8;
    return planes > kMaxPlanes ? kMaxPlanes : planes;
}

template <int OUT, int HT>
inline void launch_conv_shared_mfma_out(const SharedParams& p, int planes, dim3 grid, hipStream_t stream)
{
    const dim3 block(256);
    switch (planes) {
        case 1: hipLaunchKernelGGL((k_conv_shared_mfma<1, OUT, HT>), grid, block, 0, stream, p); break;
        case 2: hipLaunchKernelGGL((k_conv_shared_mfma<2, OUT, HT>), grid, block, 0, stream, p); break;
        case 3: hipLaunchKernelGGL((k_conv_shared_mfma<3, OUT, HT>), grid, block, 0, stream, p); break;
        default: hipLaunchKernelGGL((k_conv_shared_mfma<4, OUT, HT>), grid, block, 0, stream, p); break;
    }
}

template <int OUT, int HT>
inline void launch_conv_shared_mfma_resident(const SharedParams& p, int planes, dim3 grid, unsigned columns, size_t lds,
                                             hipStream_t stream)
{
    const dim3 block(256);
    switch (planes) {
        case 1: hipLaunchKernelGGL((k_conv_shared_mfma_resident<1, OUT, HT>), grid, block, lds, stream, p, columns); break;
        case 2: hipLaunchKernelGGL((k_conv_shared_mfma_resident<2, OUT, HT>), grid, block, lds, stream, p, columns); break;
        case 3: hipLaunchKernelGGL((k_conv_shared_mfma_resident<3, OUT, HT>), grid, block, lds, stream, p, columns); break;
        default: hipLaunchKernelGGL((k_conv_shared_mfma_resident<4, OUT, HT>), grid, block, lds, stream, p, columns); break;
    }
}

// Whether k_conv3x3_window can take the call, and in which shape.  slots = the longest window of a pixel tile:
// T - 1 positions between its first and last pixel, one more per image row and W + 1 more per image that the tile
// crosses, and the taps' reach of 2 (W + 1) + 2 beyond the last pixel.
struct WindowPlan { bool ok; int teams, ws; };
// slots of the longest window of a layer with this geometry, or 0 when the kernel does not take the geometry
// (the reduction of such a layer is never split over workgroups: the teams do that inside one)
inline int window_slots(int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w, int H, int W, int half_tiles)
{
    static const bool enabled = [] { const char* v = std::getenv("PSB_SHARED_WINDOW"); return !(v && std::atoi(v) == 0); }();   // benchmark switch
    if (!enabled || kh != 3 || kw != 3 || stride_h != 1 || stride_w != 1 || pad_h != 1 || pad_w != 1) return 0;
    const int64_t T = 128 * half_tiles;
    const int64_t rows = (T + W - 2) / W, images = (T + (int64_t)H * W - 2) / ((int64_t)H * W);
    const int64_t slots = T - 1 + rows + images * (W + 1) + 2 * (W + 1) + 3;
    return slots <= 512 ? (int)slots : 0;
}
inline WindowPlan window_plan(const SharedParams& p, int planes, int half_tiles, int n_cus)
{
    WindowPlan w{false, 1, 1};
    if (p.OH != p.tH || p.OW != p.tW || p.ksplit != 1 || planes < 3) return w;
    const int64_t T = 128 * half_tiles;
    const int slots = window_slots(p.tKH, p.tKW, p.t_stride_h, p.t_stride_w, p.t_pad_h, p.t_pad_w, p.tH, p.tW, half_tiles);
    if (slots == 0) return w;
    w.ws = slots <= 256 ? 1 : 2;
    if (half_tiles == 2 && w.ws != 2) return w;      // (cannot happen: 256 pixels need more than 256 slots)
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    const int64_t wgs = (npix + T - 1) / T * ((p.OC + 31) / 32);
    const int CB = p.C_pad >> 5;
    // two teams when the layer has at most one workgroup per CU: then every SIMD still gets two waves
    w.teams = (half_tiles == 1 && CB % 2 == 0 && CB >= 4 && wgs <= n_cus) ? 2 : 1;
    w.ok = true;
    return w;
}

template <int P, int OUT, int HT, int TEAMS, int WS>
inline bool launch_window_one(const SharedParams& p, dim3 grid, hipStream_t stream)
{
    constexpr int kAregs = (9 * P * 64 + 255) / 256;
    constexpr size_t lds = (size_t)TEAMS * (kAregs + 2 * WS) * 4096;
    static_assert(TEAMS == 1 || (size_t)(TEAMS - 1) * 4 * HT * P * 4 * 64 * 16 <= lds, "the teams' sums must fit the operand area");
    auto kernel = k_conv3x3_window<P, OUT, HT, TEAMS, WS>;
    // more than 64 KB of dynamic LDS has to be asked for once
    static const bool usable = lds <= 65536 || hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
    if (!usable) return false;
    hipLaunchKernelGGL(kernel, grid, dim3(256 * TEAMS), lds, stream, p);
    return true;
}

template <int P, int OUT>
inline bool launch_window_shape(const SharedParams& p, int half_tiles, const WindowPlan& w, dim3 grid, hipStream_t stream)
{
    if (half_tiles == 2) return launch_window_one<P, OUT, 2, 1, 2>(p, grid, stream);
    if (w.teams == 2) return w.ws == 1 ? launch_window_one<P, OUT, 1, 2, 1>(p, grid, stream) : launch_window_one<P, OUT, 1, 2, 2>(p, grid, stream);
    return w.ws == 1 ? launch_window_one<P, OUT, 1, 1, 1>(p, grid, stream) : launch_window_one<P, OUT, 1, 1, 2>(p, grid, stream);
}

template <int OUT>
inline bool launch_window_out(const SharedParams& p, int planes, int half_tiles, const WindowPlan& w, dim3 grid, hipStream_t stream)
{
    return planes == 3 ? launch_window_shape<3, OUT>(p, half_tiles, w, grid, stream) : launch_window_shape<4, OUT>(p, half_tiles, w, grid, stream);
}

// Half tiles (32 pixels) per wave: two, unless the layer is so small that one-half-tile waves still fit the chip at
// once (then twice the waves share the work, and a long reduction need not be split).
inline int shared_half_tiles(int64_t npix, int n_ocb) { return (npix + 63) / 64 * n_ocb <= 1024 ? 1 : 2; }

// resident_wgs: workgroups the chip holds at once with this kernel (two per CU), or 0 to rule the persistent variant out.
// half_tiles: shared_half_tiles() of the layer (p.ksplit was chosen for it).
inline void launch_conv_shared_mfma(const SharedParams& p, int planes, int resident_wgs, int half_tiles, hipStream_t stream)
{
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    const int64_t wg_pixels = 128 * half_tiles;
    const int64_t tiles = (npix + wg_pixels - 1) / wg_pixels;
    const unsigned columns = (unsigned)((tiles + 7) / 8 * 8);                        // 8 XCDs
    const unsigned n_ocb = (unsigned)((p.OC + 31) / 32);
    const int n_steps = p.tKH * p.tKW * (p.C_pad >> 5);
    const size_t lds = (size_t)n_steps * planes * kPlaneStride;
    const WindowPlan win = window_plan(p, planes, half_tiles, std::max(resident_wgs, 512) / 2);
    if (win.ok) {
        SharedParams pw = p;
        // weights (digit planes) against activations, in bytes: worth it from about twice as many on (measured)
        pw.xcd_by_channels = n_ocb % 8 == 0 && (int64_t)n_ocb * 32 * n_steps * 32 * planes > 2 * (int64_t)p.N * p.tH * p.tW * p.C_pad;
        const dim3 grid(pw.xcd_by_channels ? (unsigned)tiles : columns, n_ocb);
        const bool done = p.masked ? launch_window_out<kOutPartial>(pw, planes, half_tiles, win, grid, stream)
                        : p.rq.x_out ? launch_window_out<kOutRequant>(pw, planes, half_tiles, win, grid, stream)
                                     : launch_window_out<kOutAcc>(pw, planes, half_tiles, win, grid, stream);
        if (done) return;
    }
    // worth it when a workgroup gets more than one tile: staging the whole block before the first matrix instruction
    // costs more than the chunked start of the plain kernel
    const unsigned fit = std::max(8u, (unsigned)std::max(resident_wgs, 0) / n_ocb / 8u * 8u);
    if (half_tiles == 2 && resident_wgs > 0 && !p.masked && p.n_seg == 0 && p.ksplit == 1 && lds <= 65536 && columns > fit) {
        // A short reduction leaves the walk bound by the vector instructions of tile set-up and epilogue (the first
        // convolution of a ResNet: ~1000 per tile and wave against 42 matrix instructions), which two waves per SIMD
        // issue at half the rate four do: one half tile per wave then (half the accumulators, four waves per SIMD),
        // when four workgroups' weight blocks fit the LDS of a CU (first convolution of config 4: 45 -> 37 us).
        if (lds <= 36864) {
            const unsigned columns1 = (unsigned)(((npix + 127) / 128 + 7) / 8 * 8);
            const unsigned fit1 = std::max(8u, 2u * (unsigned)resident_wgs / n_ocb / 8u * 8u);
            const dim3 grid(std::min(fit1, columns1), n_ocb);
            if (p.rq.x_out) launch_conv_shared_mfma_resident<kOutRequant, 1>(p, planes, grid, columns1, lds, stream);
            else launch_conv_shared_mfma_resident<kOutAcc, 1>(p, planes, grid, columns1, lds, stream);
            return;
        }
        const dim3 grid(fit, n_ocb);
        if (p.rq.x_out) launch_conv_shared_mfma_resident<kOutRequant, 2>(p, planes, grid, columns, lds, stream);
        else launch_conv_shared_mfma_resident<kOutAcc, 2>(p, planes, grid, columns, lds, stream);
        return;
    }
    const dim3 grid(columns, n_ocb, (unsigned)p.ksplit);
    if (half_tiles == 1) {
        if (p.masked || p.ksplit > 1) launch_conv_shared_mfma_out<kOutPartial, 1>(p, planes, grid, stream);
        else if (p.rq.x_out) launch_conv_shared_mfma_out<kOutRequant, 1>(p, planes, grid, stream);
        else launch_conv_shared_mfma_out<kOutAcc, 1>(p, planes, grid, stream);
    } else {
        if (p.masked || p.ksplit > 1) launch_conv_shared_mfma_out<kOutPartial, 2>(p, planes, grid, stream);
        else if (p.rq.x_out) launch_conv_shared_mfma_out<kOutRequant, 2>(p, planes, grid, stream);
        else launch_conv_shared_mfma_out<kOutAcc, 2>(p, planes, grid, stream);
    }
}

}  // namespace psb
