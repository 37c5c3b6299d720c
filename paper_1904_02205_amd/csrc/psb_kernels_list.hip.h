// "Product-list" layer kernel: any layer shape, made for the ones the channel-lane kernel cannot
// serve well - grouped and depthwise convolutions, and layers whose weights are mostly pruned.
//
// A workgroup owns one output channel and 256 consecutive output pixels.  For a chunk of up to 10 LIVE
// taps of that channel (a per-channel index of live taps is built when the weights are encoded, so dead
// weights cost nothing) it first builds, in LDS, the list of all products that need sampling - live
// weight, tap inside the image, activation != 0 - by ballot/prefix compaction over the pixels, then the
// 256 lanes take list entries round-robin, sample them, and add the result to the pixel's accumulator in
// LDS (ds_add, exact in any order).  Every lane therefore always has a product to work on, whatever the
// sparsity pattern.  Output index and tap differ per lane, so the parts of the first three generator
// rounds that depend on only one of the two cannot stay in registers; for calls with the same S everywhere
// (up to four generator blocks) they are kept in two LDS tables instead - one row per pixel, one per tap
// of the chunk - and a call costs 15 wide multiplies as in the channel-lane kernel; the other calls run
// the whole generator per entry (19 multiplies).  No global atomics, no zero-fill: the accumulators leave
// LDS once, with the fp32 epilogue fused.
// The chunk is short on purpose: the list is the largest LDS array, and with 10 taps (23 KB per workgroup
// with the tables) seven workgroups share a compute unit, whose waves hide each other's list building,
// table loads and barriers; 24- and 32-tap chunks (4 and 3 workgroups) measured 10 % slower.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "psb_kernels.hip.h"
#include "psb_kernels_oc.hip.h"

namespace psb {

constexpr int kListPixels = 256;                       // pixels per workgroup = threads per workgroup
constexpr int kListTaps = 10;                          // live taps per chunk
constexpr int kListCap = kListPixels * kListTaps;      // list entries

// live_idx[oc][0 .. live_cnt[oc]) = taps k of channel oc whose weight is sampled (any order).
// One workgroup per output channel.
__global__ void __launch_bounds__(256) k_live_index(const uint32_t* __restrict__ packed, int K,
                                                    uint32_t* __restrict__ live_idx, uint32_t* __restrict__ live_cnt)
{
    __shared__ uint32_t count;
    if (threadIdx.x == 0) count = 0;
    __syncthreads();
    const int oc = blockIdx.x;
    const int lane = threadIdx.x & 63;
    for (int k0 = 0; k0 < K; k0 += 256) {
        const int k = k0 + threadIdx.x;
        const bool live = k < K && (packed[(int64_t)oc * K + k] & 0x7F800000u) != kDeadWord;
        const unsigned long long mask = __ballot(live);
        uint32_t base = 0;
        if (lane == 0 && mask) base = atomicAdd(&count, (uint32_t)__popcll(mask));
        base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
        if (live) {
            const uint32_t pos = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                  __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            live_idx[(int64_t)oc * K + pos] = (uint32_t)k;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) live_cnt[oc] = count;
}

// Samples of block j of product (o, k) that are below thr; all arguments per lane.
__device__ __forceinline__ uint32_t count_block_full(uint32_t o, uint32_t k, uint32_t j, uint32_t layer, uint32_t key0,
                                                     uint32_t key1, uint32_t thr)
{
    const u32x4 r = philox4x32_10(u32x4{o, k, j, layer}, key0, key1);
    return (r.x < thr ? 1u : 0u) + (r.y < thr ? 1u : 0u) + (r.z < thr ? 1u : 0u) + (r.w < thr ? 1u : 0u);
}

// Same with sixteen 7-bit uniforms per block, thr4 = the 7-bit threshold in each byte.
__device__ __forceinline__ uint32_t count_block_full7(uint32_t o, uint32_t k, uint32_t j, uint32_t layer, uint32_t key0,
                                                      uint32_t key1, uint32_t thr4)
{
    const u32x4 r = philox4x32_10(u32x4{o, k, j, layer}, key0, key1);
    const uint32_t all = 0x80808080u;
    return 16u - (not_below7(r.x, thr4, all) + not_below7(r.y, thr4, all) + not_below7(r.z, thr4, all) +
                  not_below7(r.w, thr4, all));
}

// NB > 0: every pixel draws the samples of generator blocks 0 .. NB-1, all of them (a call with the
//         same S everywhere, S = NB * samples per block).
// NB = 0: per-pixel ranges [from, to), any values.
// P7: 7-bit uniforms, 16 samples per block; otherwise 32-bit uniforms, 4 per block.
// INSIDE: every tap of every output pixel lies inside the image (1 x 1 layers, unpadded layers): no bounds checks.
template <int NB, bool P7, bool INSIDE>
__global__ void __launch_bounds__(kListPixels, 7) k_layer_product_list(const LayerParams p,
                                                                    const uint32_t* __restrict__ live_idx,
                                                                    const uint32_t* __restrict__ live_cnt,
                                                                    int channels_per_wg)
{
    // HOIST: the tap-independent and the pixel-independent parts of generator rounds 0..2 come from tables
    constexpr bool HOIST = NB >= 1 && NB <= 4;
    constexpr int NBT = HOIST ? NB : 1;
    __shared__ uint32_t list[kListCap];          // pixel | tap slot << 8 | activation byte << 16
    __shared__ int32_t acc_s[kListPixels];
    __shared__ uint32_t o_s[HOIST ? 1 : kListPixels];      // flat output index of the pixel for this channel
    __shared__ uint32_t range_s[kListPixels];    // from | to << 8
    __shared__ uint32_t ktab[kListTaps];         // tap index k
    __shared__ uint2 wtab[kListTaps];            // {threshold, +-2^shift}
    __shared__ int2 tapinfo[kListTaps];          // {offset inside the image group, kh | kw << 16}
    __shared__ uint2 pix_base[HOIST ? kListPixels : 1];    // per pixel: {low half of MulA * o, state word 1 after round 1 ^ key}
    __shared__ __align__(16) uint2 pix_blk[HOIST ? kListPixels : 1][NBT];   // per (pixel, block): round 2's MulA product
    __shared__ __align__(16) uint2 tap_blk[HOIST ? kListTaps : 1][NBT];     // per (tap, block): round 1's MulA product
    __shared__ uint32_t count;

    Keys key;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        key.k0[r] = p.key0 + (uint32_t)r * kWeyl0;
        key.k1[r] = p.key1 + (uint32_t)r * kWeyl1;
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    const int64_t pix = (int64_t)blockIdx.x * kListPixels + tid;
    const bool valid = pix < npix;
    const int64_t pixc = valid ? pix : npix - 1;
    const uint32_t pix32 = (uint32_t)pixc;                 // the number of outputs fits 32 bits, so pixels do too
    const uint32_t row32 = pix32 / (uint32_t)p.OW;
    const int ox = (int)(pix32 - row32 * (uint32_t)p.OW);
    const int n = (int)(row32 / (uint32_t)p.OH);
    const int oy = (int)(row32 - (uint32_t)n * (uint32_t)p.OH);
    int to = p.budget_to ? (int)p.budget_to[pixc] : p.S;
    to = min(to, p.s_max);
    int from = p.budget_from ? (int)p.budget_from[pixc] : 0;
    from = min(from, to);
    const int iy0 = oy * p.stride_h - p.pad_h;
    const int ix0 = ox * p.stride_w - p.pad_w;
    const bool wants = valid && to > from;
    range_s[tid] = (uint32_t)from | ((uint32_t)to << 8);

    // the whole activation tensor as a raw buffer (stride 0, size in bytes below 2^31, 32-bit data format)
    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t*>(p.x), 0, (int)((int64_t)p.N * p.C * p.H * p.W), 0x00020000);
    if (tid < kListTaps) tapinfo[tid] = make_int2(0, 0);     // every row is a tap of this geometry from the start
    constexpr uint32_t kBeyond = 0x80000000u;                // an offset no tensor reaches

    // A workgroup serves channels_per_wg consecutive channels one after the other, so that the per-pixel set-up
    // above is paid once even when a channel has only a handful of taps (depthwise layers).
    const int oc_end = min(p.OC, ((int)blockIdx.y + 1) * channels_per_wg);
    for (int oc = (int)blockIdx.y * channels_per_wg; oc < oc_end; ++oc) {
    const uint32_t o = (uint32_t)((((int64_t)n * p.OC + oc) * p.OH + oy) * p.OW + ox);
    const int grp = oc / p.OCg;
    // index of x[n][grp*Cg][iy0][ix0] modulo 2^32; only dereferenced with an in-bounds tap offset added
    const uint32_t xbase = (uint32_t)((((int64_t)n * p.C + (int64_t)grp * p.Cg) * p.H + iy0) * p.W + ix0);

    acc_s[tid] = 0;
    if constexpr (HOIST) {
        // rounds 0..2 of this pixel's counter, as far as they go without the tap
        PixelHoist h;
        uint32_t hi_a, lo_b1;
        mulhilo(kMulA, o, hi_a, h.lo_a);
        mulhilo(kMulB, hi_a ^ p.layer_id ^ key.k1[0], h.hi_b1, lo_b1);
        h.y2k = lo_b1 ^ key.k0[2];
        pix_base[tid] = make_uint2(h.lo_a, h.y2k);
#pragma unroll
        for (int j = 0; j < NBT; ++j) {
            uint32_t s_hib, hz, lo2;
            block_setup(h, key, j, s_hib, hz, lo2);
            pix_blk[tid][j] = make_uint2(hz, lo2);
        }
    } else {
        o_s[tid] = o;
    }

    const uint32_t nlive = live_cnt[oc];
    for (uint32_t c0 = 0; c0 < nlive; c0 += kListTaps) {
        const int nk = (int)min((uint32_t)kListTaps, nlive - c0);
        if (tid < nk) {
            const uint32_t k = live_idx[(int64_t)oc * p.K + c0 + tid];
            const uint32_t word = p.packed[(int64_t)oc * p.K + k];
            const uint32_t unit = 1u << ((word >> 23) & 0xFFu);
            ktab[tid] = k;
            wtab[tid] = make_uint2(threshold_of(word & 0x7FFFFFu, P7 ? 7 : 23), (word & 0x80000000u) ? (0u - unit) : unit);
            const int khw = p.KH * p.KW;
            const int ci = (int)k / khw;
            const int r = (int)k - ci * khw;
            const int kh = r / p.KW;
            const int kw = r - kh * p.KW;
            tapinfo[tid] = make_int2((ci * p.H + kh) * p.W + kw, kh | (kw << 16));
            if constexpr (HOIST) {
#pragma unroll
                for (int j = 0; j < NBT; ++j) {
                    uint32_t hi_bj, lo_bj;
                    mulhilo(kMulB, (uint32_t)j, hi_bj, lo_bj);
                    const TapScalars ts = tap_scalars(hi_bj ^ key.k0[0] ^ k, key);
                    tap_blk[tid][j] = make_uint2(ts.sz, ts.s_lo);
                }
            }
        }
        if (tid == 0) count = 0;
        __syncthreads();

        // Build the list of products that need sampling.  First every lane requests the activations of all taps
        // of the chunk (independent loads: one memory latency for the lot), then each wave compacts its own
        // entries: one range of the list is reserved per wave with a single LDS atomic, and positions inside the
        // range follow from ballots and prefix counts.  (The order of the list is irrelevant to the result.)
        // The loads are straight-line code: a range-checked buffer load returns zero for an offset beyond the
        // tensor, which is what a tap outside the image gets, so no load waits for a branch or for another load.
        // Table rows beyond nk hold taps of an earlier chunk: their loads are harmless, their values not looked at.
        uint32_t xv[kListTaps];
        if constexpr (INSIDE) {      // only lanes without work need the out-of-range offset
            const uint32_t from_here = wants ? xbase : kBeyond;      // kBeyond + a tap offset stays beyond the tensor
#pragma unroll
            for (int i = 0; i < kListTaps; ++i)
                xv[i] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(x_rsrc, (int)(from_here + (uint32_t)tapinfo[i].x), 0, 0);
        } else {
#pragma unroll
            for (int i = 0; i < kListTaps; ++i) {
                const int2 info = tapinfo[i];
                const int iy = iy0 + (info.y & 0xFFFF);
                const int ix = ix0 + (info.y >> 16);
                const bool ok = wants & ((unsigned)iy < (unsigned)p.H) & ((unsigned)ix < (unsigned)p.W);   // no branches
                // the index of an element that exists is below 2^31, so 32-bit arithmetic modulo 2^32 finds it
                const uint32_t at = ok ? xbase + (uint32_t)info.x : kBeyond;
                xv[i] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(x_rsrc, (int)at, 0, 0);
            }
        }
        uint32_t mine = 0;           // entries of this wave (uniform)
#pragma unroll
        for (int i = 0; i < kListTaps; ++i)
            if (i < nk) mine += (uint32_t)__popcll(__ballot(xv[i] != 0));
        uint32_t run = 0;
        if (lane == 0 && mine) run = atomicAdd(&count, mine);
        run = (uint32_t)__builtin_amdgcn_readfirstlane((int)run);
#pragma unroll
        for (int i = 0; i < kListTaps; ++i) {
            if (i < nk) {
                const unsigned long long mask = __ballot(xv[i] != 0);
                if (xv[i] != 0) {
                    const uint32_t pos = run + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                    list[pos] = (uint32_t)tid | ((uint32_t)i << 8) | (xv[i] << 16);
                }
                run += (uint32_t)__popcll(mask);
            }
        }
        __syncthreads();

        // sample the products, lanes taking entries round-robin
        const uint32_t total = count;
        if constexpr (NB > 0) {
            constexpr int U = (NB >= 4) ? 1 : 4 / NB;      // entries in flight per lane: four independent calls
            for (uint32_t e0 = (uint32_t)tid; e0 < total; e0 += (uint32_t)(U * kListPixels)) {
                uint32_t cnt[U];
                uint32_t ent[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t e = e0 + (uint32_t)(u * kListPixels);
                    ent[u] = (e < total) ? list[e] : 0xFFFFFFFFu;
                    cnt[u] = 0;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (ent[u] == 0xFFFFFFFFu) continue;
                    const uint32_t slot = (ent[u] >> 8) & 0xFFu;
                    const uint32_t thr = wtab[slot].x;
                    if constexpr (HOIST) {
                        const uint32_t pl = ent[u] & 0xFFu;
                        const uint2 base = pix_base[pl];
                        const PixelHoist h{base.x, 0u, base.y};
#pragma unroll
                        for (int j = 0; j < NB; ++j) {
                            const uint2 pb = pix_blk[pl][j];
                            const uint2 tb = tap_blk[slot][j];
                            cnt[u] += sample_block<4, P7>(thr, TapScalars{tb.x, tb.y}, h, pb.x, pb.y, key, j, 0, 0);
                        }
                    } else {
                        const uint32_t ou = o_s[ent[u] & 0xFFu];
                        const uint32_t ku = ktab[slot];
#pragma unroll
                        for (int j = 0; j < NB; ++j)
                            cnt[u] += P7 ? count_block_full7(ou, ku, (uint32_t)j, p.layer_id, p.key0, p.key1, thr)
                                         : count_block_full(ou, ku, (uint32_t)j, p.layer_id, p.key0, p.key1, thr);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (ent[u] == 0xFFFFFFFFu) continue;
                    const int32_t xs = (int32_t)(int8_t)((ent[u] >> 16) & 0xFFu);
                    const int32_t unit = (int32_t)wtab[(ent[u] >> 8) & 0xFFu].y;
                    const int32_t term = (int32_t)((uint32_t)xs * ((uint32_t)((P7 ? 16 : 4) * NB) + cnt[u]) * (uint32_t)unit);   // modulo 2^32
                    atomicAdd(&acc_s[ent[u] & 0xFFu], term);
                }
            }
        } else {
            for (uint32_t e = (uint32_t)tid; e < total; e += (uint32_t)kListPixels) {
                const uint32_t entry = list[e];
                const uint32_t pl = entry & 0xFFu;
                const uint32_t slot = (entry >> 8) & 0xFFu;
                const uint32_t rg = range_s[pl];
                const int f = (int)(rg & 0xFFu), t = (int)(rg >> 8);
                const uint32_t c = P7 ? count_below7(o_s[pl], ktab[slot], p.layer_id, p.key0, p.key1, wtab[slot].x, f, t)
                                      : count_below(o_s[pl], ktab[slot], p.layer_id, p.key0, p.key1, wtab[slot].x, f, t);
                const int32_t xs = (int32_t)(int8_t)((entry >> 16) & 0xFFu);
                const int32_t term = (int32_t)((uint32_t)xs * ((uint32_t)(t - f) + c) * wtab[slot].y);   // modulo 2^32
                atomicAdd(&acc_s[pl], term);
            }
        }
        __syncthreads();   // the tables and the list are rewritten by the next chunk
    }
    __syncthreads();       // acc_s is complete (also when the channel has no live tap at all)

    if (valid) {
        int32_t total = acc_s[tid];
        if (p.budget_from) total += p.acc[o];
        if (p.acc) p.acc[o] = total;
        emit(p, o, oc, total, to);
    }
    }   // channels of this workgroup (acc_s and o_s are only touched by their own lane between the barriers)
}

// Returns 0 or a hipError_t.
inline int launch_product_list(const LayerParams& p, const uint32_t* live_idx, const uint32_t* live_cnt,
                               hipStream_t stream, bool (*prof_begin)(hipStream_t, int*),
                               void (*prof_end)(hipStream_t, int))
{
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    const int64_t gx = (npix + kListPixels - 1) / kListPixels;
    // enough channels per workgroup for about 64 taps of work per pixel, at most 8
    const int channels_per_wg = (int)std::min<int64_t>(8, std::max<int64_t>(1, 64 / std::max(1, p.K)));
    const int gy = (p.OC + channels_per_wg - 1) / channels_per_wg;
    if (gx > 2147483647ll || gy > 65535) return (int)hipErrorInvalidValue;
    const dim3 grid((unsigned)gx, (unsigned)gy), block(kListPixels);
    // compile-time block count only for a uniform S that is a whole number of generator blocks
    const bool p7 = p.prob_bits <= 7;
    const int per_block = p7 ? 16 : 4;
    int nb = 0;
    if (!p.budget_to && p.S % per_block == 0) nb = p.S / per_block;
    int slot = 0;
    const bool timed = prof_begin(stream, &slot);
    const bool inside = p.pad_h == 0 && p.pad_w == 0 && (int64_t)(p.OH - 1) * p.stride_h + p.KH <= p.H &&
                        (int64_t)(p.OW - 1) * p.stride_w + p.KW <= p.W;
#define PSB_LAUNCH(NB_, P7_)                                                                                      \
    do {                                                                                                          \
        if (inside)                                                                                               \
            hipLaunchKernelGGL((k_layer_product_list<NB_, P7_, true>), grid, block, 0, stream, p, live_idx,       \
                               live_cnt, channels_per_wg);                                                        \
        else                                                                                                      \
            hipLaunchKernelGGL((k_layer_product_list<NB_, P7_, false>), grid, block, 0, stream, p, live_idx,      \
                               live_cnt, channels_per_wg);                                                        \
    } while (0)
    if (p7) {
        switch (nb) {
            case 1: PSB_LAUNCH(1, true); break;
            case 2: PSB_LAUNCH(2, true); break;
            default: PSB_LAUNCH(0, true); break;
        }
    } else {
        switch (nb) {
            case 1: PSB_LAUNCH(1, false); break;
            case 2: PSB_LAUNCH(2, false); break;
            case 4: PSB_LAUNCH(4, false); break;
            case 8: PSB_LAUNCH(8, false); break;
            default: PSB_LAUNCH(0, false); break;
        }
    }
#undef PSB_LAUNCH
    if (timed) prof_end(stream, slot);
    return (int)hipGetLastError();
}

}  // namespace psb
