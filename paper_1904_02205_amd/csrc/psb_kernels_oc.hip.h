// "Channel-lane" layer kernel for dense layers with groups = 1 (gfx950, wave64).
//
// Mapping: lane = output channel inside a block of 64, wave = one output pixel at a
// time.  The activation of a tap is then the same for all lanes, so
//   - taps whose activation is 0 (about half after a ReLU, and all padding) are removed
//     before the sampling loop by a wave-level compaction (ballot + prefix count) into a
//     per-wave list in LDS: no lane ever idles on a zero product;
//   - the sample range [from,to) of a progressive call is wave-uniform: no divergence;
//   - everything of the Philox counter that depends on the tap only is scalar work.
// The weights of one tile of taps x 64 channels are staged in LDS once per workgroup as
// {threshold, +-2^shift} pairs and read conflict-free (one ds_read_b64 per product).
//
// The reduction over taps is split into chunks; with more than one chunk the partial
// sums are combined with int32 atomic adds, which is exact in any order because the
// accumulator arithmetic is modulo 2^32.  They meet in scratch accumulators laid out
// [N*OH*OW][OC padded to 64], where the 64 adds of a wave are consecutive words; a last
// pass turns them into the [N][OC][OH][OW] outputs.
//
// Philox work saved without changing a bit of the result.  Counter = (o, k, j, layer).
// Round 0 multiplies o and j; o is fixed per lane and pixel, j is a literal.  Round 1
// multiplies a scalar (a function of k and j) and a per-lane value that depends on o
// only.  Round 2 multiplies a value that depends on (o, j) only and one that depends on
// everything.  So of the 20 wide multiplies of a call only 15 are per-product vector
// work; the other five are hoisted to per-pixel set-up or to the scalar unit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdlib>

#include "psb_kernels.hip.h"

namespace psb {

constexpr int kOcWaves = 4;     // waves per workgroup
constexpr int kOcMaxTaps = 64;  // taps per LDS tile: 64 * 64 channels * 8 B = 32 KB

__device__ __forceinline__ uint32_t uniform_u32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

// a*b + c with 24-bit signed a, b (full-rate v_mad_i32_i24)
__device__ __forceinline__ int32_t mad24(int32_t a, int32_t b, int32_t c) { return __mul24(a, b) + c; }

struct PixelHoist {
    uint32_t lo_a;    // low half of MulA * o                          (round 0, word 3)
    uint32_t hi_b1;   // high half of MulB * (state word 2 after round 0)
    uint32_t y2k;     // low half of the same product, xor round-2 key 0
};

// Round keys and multipliers.  Everything here is wave-uniform and stays in scalar registers.  (An instruction
// stream in which EVERY two-operand VALU instruction has a scalar-register source issues at half rate on gfx950 -
// 4.2 vs 2.4 cycles per wave64 - but in this loop only the key xors and the multiplies by the two constants have
// one, and copies of the keys (16 registers) or of the two multipliers in vector registers measured no gain.)
struct Keys {
    uint32_t k0[10], k1[10];
};

// Rounds 3..9.
__device__ __forceinline__ u32x4 philox_rounds_3_to_9(u32x4 c, const Keys& key)
{
#pragma unroll
    for (int r = 0; r < 7; ++r) {
        uint32_t hi_a, lo_a, hi_b, lo_b;
        mulhilo(kMulA, c.x, hi_a, lo_a);
        mulhilo(kMulB, c.z, hi_b, lo_b);
        u32x4 t;
        t.x = hi_b ^ c.y ^ key.k0[r + 3];
        t.y = lo_b;
        t.z = hi_a ^ c.w ^ key.k1[r + 3];
        t.w = lo_a;
        c = t;
    }
    return c;
}

// Scalar half of round 1 for one (tap, block): word 0 of the state after round 0 is s_x1 = s_hib ^ k.
// Returns the two scalars the vector part needs.
struct TapScalars { uint32_t sz, s_lo; };
__device__ __forceinline__ TapScalars tap_scalars(uint32_t s_x1, const Keys& key)
{
    uint32_t s_hi, s_lo;
    mulhilo(kMulA, s_x1, s_hi, s_lo);
    return TapScalars{s_hi ^ key.k1[1], s_lo};
}

// Number of samples of block j of one product that are below thr.  P7: the block holds sixteen 7-bit
// uniforms and thr the 7-bit threshold in each byte; otherwise four 32-bit uniforms.
// VALID = 4: every sample of the block counts; 1..3: the first VALID samples count with 32-bit uniforms, the first
// 4 VALID (whole words) with 7-bit uniforms (the last block of a range that starts on a block boundary);
// 0: the range [from,to) is checked at run time.
// state after round 1: (.., .., ts.sz ^ lo_a, ts.s_lo); words 0 and 1 were used in the per-pixel set-up.
template <int VALID, bool P7>
__device__ __forceinline__ uint32_t sample_block(uint32_t thr, TapScalars ts, const PixelHoist& h, uint32_t hz,
                                                 uint32_t lo2, const Keys& key, int j, int from, int to)
{
    const uint32_t z2 = ts.sz ^ h.lo_a;
    // round 2: only MulB * z2 is new
    uint32_t hi_b2, lo_b2;
    mulhilo(kMulB, z2, hi_b2, lo_b2);
    u32x4 c;
    c.x = hi_b2 ^ h.y2k;
    c.y = lo_b2;
    c.z = hz ^ ts.s_lo;
    c.w = lo2;
    c = philox_rounds_3_to_9(c, key);
    uint32_t n = 0;
    if constexpr (P7) {
        if constexpr (VALID > 0) {       // the first 4 VALID samples of the block: its first VALID words, whole
            const uint32_t all = 0x80808080u;
            uint32_t not_below = not_below7(c.x, thr, all);
            if (VALID > 1) not_below += not_below7(c.y, thr, all);
            if (VALID > 2) not_below += not_below7(c.z, thr, all);
            if (VALID > 3) not_below += not_below7(c.w, thr, all);
            return (uint32_t)(4 * VALID) - not_below;
        }
        const int lo = max(from, 16 * j), hi = min(to, 16 * j + 16);
        return (uint32_t)(hi - lo) -
               (not_below7(c.x, thr, valid_bytes7(j, 0, from, to)) + not_below7(c.y, thr, valid_bytes7(j, 1, from, to)) +
                not_below7(c.z, thr, valid_bytes7(j, 2, from, to)) + not_below7(c.w, thr, valid_bytes7(j, 3, from, to)));
    } else if constexpr (VALID > 0) {
        n += (c.x < thr) ? 1u : 0u;
        if (VALID > 1) n += (c.y < thr) ? 1u : 0u;
        if (VALID > 2) n += (c.z < thr) ? 1u : 0u;
        if (VALID > 3) n += (c.w < thr) ? 1u : 0u;
    } else {
        const int s0 = 4 * j;
        n += (s0 + 0 >= from && s0 + 0 < to && c.x < thr) ? 1u : 0u;
        n += (s0 + 1 >= from && s0 + 1 < to && c.y < thr) ? 1u : 0u;
        n += (s0 + 2 >= from && s0 + 2 < to && c.z < thr) ? 1u : 0u;
        n += (s0 + 3 >= from && s0 + 3 < to && c.w < thr) ? 1u : 0u;
    }
    return n;
}

// Per-(pixel, block j) set-up: the part of rounds 0..2 that does not depend on the tap.
__device__ __forceinline__ void block_setup(const PixelHoist& h, const Keys& key, int j, uint32_t& s_hib /* scalar */,
                                            uint32_t& hz, uint32_t& lo2)
{
    uint32_t hi_bj, lo_bj;
    mulhilo(kMulB, (uint32_t)j, hi_bj, lo_bj);          // round 0: MulB * j (scalar)
    s_hib = hi_bj ^ key.k0[0];                          // state word 0 after round 0 is s_hib ^ k
    const uint32_t x2 = h.hi_b1 ^ lo_bj ^ key.k0[1];    // state word 0 after round 1
    uint32_t hi_a2, lo_a2;
    mulhilo(kMulA, x2, hi_a2, lo_a2);                   // round 2: MulA * x2
    hz = hi_a2 ^ key.k1[2];
    lo2 = lo_a2;
}

// Entry i of the wave's compacted tap list; the list lives in one VGPR (lane i = entry i).
__device__ __forceinline__ uint32_t list_entry(uint32_t mylist, int i)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)mylist, i);
}

// All products of one pixel's compacted tap list, NB generator blocks per product
// (NB = 0: run-time number of blocks).  Returns this lane's partial accumulator.
// mylist: lane i holds entry i = (tap index inside the tile << 8) | activation byte, and 0
// beyond cnt (entry 0 addresses tile row 0, so reading one group ahead is always in bounds).
// VALID: see sample_block; with NB > 1 it applies to every block (only 4 is used then).
template <int NB, int VALID, bool P7>
__device__ __forceinline__ int32_t process_list(uint32_t mylist, int cnt, const uint2* __restrict__ w_tile,
                                                int lane, uint32_t k0, int j0, int nb_rt, int from, int to,
                                                const PixelHoist& h, const Keys& key)
{
    const uint32_t nsamp = (uint32_t)(to - from);
    int32_t acc = 0;
    if constexpr (NB == 0) {
        for (int i = 0; i < cnt; ++i) {
            const uint32_t entry = list_entry(mylist, i);
            const uint32_t kl = entry >> 8;
            const int32_t xs = (int32_t)(int8_t)(entry & 0xFFu);
            const uint2 wt = w_tile[kl * 64 + lane];
            uint32_t n = nsamp;
            for (int jj = 0; jj < nb_rt; ++jj) {
                uint32_t s_hib, hz, lo2;
                block_setup(h, key, j0 + jj, s_hib, hz, lo2);
                n += sample_block<0, P7>(wt.x, tap_scalars(s_hib ^ (k0 + kl), key), h, hz, lo2, key, j0 + jj, from, to);
            }
            acc = mad24(__mul24(xs, (int32_t)n), (int32_t)wt.y, acc);
        }
        return acc;
    } else {
        constexpr int E = (NB >= 4) ? 1 : 4 / NB;   // products in flight: keep four generator calls independent
        uint32_t s_hib[NB], hz[NB], lo2[NB];
#pragma unroll
        for (int jj = 0; jj < NB; ++jj) block_setup(h, key, j0 + jj, s_hib[jj], hz[jj], lo2[jj]);

        // Software pipeline: while group g is sampled, the list entries of group g+1 are read, their
        // weights fetched from LDS and the scalar half of their generator calls computed.
        uint32_t ent_next[E];
        uint2 wt_next[E];
        TapScalars ts_next[E][NB];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            ent_next[e] = list_entry(mylist, e);
            wt_next[e] = w_tile[(ent_next[e] >> 8) * 64 + lane];
#pragma unroll
            for (int jj = 0; jj < NB; ++jj) ts_next[e][jj] = tap_scalars(s_hib[jj] ^ (k0 + (ent_next[e] >> 8)), key);
        }
        int i = 0;
        for (; i + E <= cnt; i += E) {
            uint2 wt[E];
            int32_t xs[E];
            TapScalars ts[E][NB];
#pragma unroll
            for (int e = 0; e < E; ++e) {
                xs[e] = (int32_t)(int8_t)(ent_next[e] & 0xFFu);
                wt[e] = wt_next[e];
#pragma unroll
                for (int jj = 0; jj < NB; ++jj) ts[e][jj] = ts_next[e][jj];
            }
#pragma unroll
            for (int e = 0; e < E; ++e) {
                ent_next[e] = list_entry(mylist, (i + E + e) & 63);
                wt_next[e] = w_tile[(ent_next[e] >> 8) * 64 + lane];
#pragma unroll
                for (int jj = 0; jj < NB; ++jj)
                    ts_next[e][jj] = tap_scalars(s_hib[jj] ^ (k0 + (ent_next[e] >> 8)), key);
            }
            // the counts of the blocks are independent of each other: no serial chain over the samples
            uint32_t cnt_b[E][NB];
#pragma unroll
            for (int e = 0; e < E; ++e)
#pragma unroll
                for (int jj = 0; jj < NB; ++jj)
                    cnt_b[e][jj] = sample_block<VALID, P7>(wt[e].x, ts[e][jj], h, hz[jj], lo2[jj], key, j0 + jj, from, to);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                uint32_t n = nsamp;
#pragma unroll
                for (int jj = 0; jj < NB; ++jj) n += cnt_b[e][jj];
                acc = mad24(__mul24(xs[e], (int32_t)n), (int32_t)wt[e].y, acc);
            }
        }
        if constexpr (E > 1) {
            for (; i < cnt; ++i) {      // fewer than E products left
                const uint32_t entry = list_entry(mylist, i);
                const uint2 wt = w_tile[(entry >> 8) * 64 + lane];
                uint32_t n = nsamp;
#pragma unroll
                for (int jj = 0; jj < NB; ++jj)
                    n += sample_block<VALID, P7>(wt.x, tap_scalars(s_hib[jj] ^ (k0 + (entry >> 8)), key), h, hz[jj], lo2[jj],
                                            key, j0 + jj, from, to);
                acc = mad24(__mul24((int32_t)(int8_t)(entry & 0xFFu), (int32_t)n), (int32_t)wt.y, acc);
            }
        }
        return acc;
    }
}

// Persistent kernel.  A ticket is one (channel block, tap chunk, group of WAVES * ppw pixels:
// ppw per wave); tickets are numbered so that consecutive tickets are consecutive pixel groups
// of the same (channel block, chunk).  Workgroups draw tickets from a device counter until none is left:
// the grid is only as large as the chip can hold at once, there is no launch gap between
// work items, and the tail at the end of the kernel is at most one ticket long.
//   sched[0] = number of tickets drawn from the counter; the launcher sets it to 0 on the stream before
//   every launch (in the kernel that zero-fills the accumulators, where there is one).
// FIXED_P7: the layer uses 7-bit uniforms (prob_bits < 23); each kernel is compiled for one of the two.
// FIXED_NB > 0: every pixel draws generator blocks 0 .. FIXED_NB-1 completely (a call with one S everywhere that is
// a whole number of blocks).  Only that path of the sampling loop is compiled then, which
// takes 76 vector registers instead of 110 and measured 3 % faster than the kernel that can do everything.
// FIXED_VALID < 4 (with FIXED_NB = 1, 7-bit uniforms): every pixel draws the first 4 FIXED_VALID samples of block 0
// (S = 4, 8 or 12: a 16-sample block is more than such a call needs).
// ppw: pixels per wave and ticket.
template <int WAVES, int FIXED_NB = 0, bool FIXED_P7 = false, int FIXED_VALID = 4>
__global__ void __launch_bounds__(WAVES * 64) k_layer_oc_lane(const LayerParams p, int n_chunks, int kc,
                                                              uint32_t pixel_groups, uint32_t n_tickets,
                                                              uint32_t* __restrict__ sched, int ppw)
{
    __shared__ uint2 w_tile[kOcMaxTaps * 64];
    __shared__ int2 tap_tab[kOcMaxTaps];
    __shared__ uint32_t lists[WAVES][kOcMaxTaps];
    __shared__ uint32_t s_ticket;

    const int lane = threadIdx.x & 63;
    const int wave = (int)uniform_u32(threadIdx.x >> 6);

    Keys key;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        key.k0[r] = p.key0 + (uint32_t)r * kWeyl0;
        key.k1[r] = p.key1 + (uint32_t)r * kWeyl1;
    }

    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    uint32_t* list = lists[wave];
    uint32_t staged = 0xFFFFFFFFu;   // (channel block, chunk) whose weights are in w_tile

    // The first ticket of a workgroup is its index (the grid never exceeds the number of tickets); only
    // later ones come from the counter, so the launch does not start with every workgroup hitting one address.
    bool first = true;
    for (;;) {
        uint32_t ticket;
        if (first) {
            ticket = blockIdx.x;
            first = false;
        } else {
            if (threadIdx.x == 0) s_ticket = gridDim.x + atomicAdd(&sched[0], 1u);
            __syncthreads();
            ticket = s_ticket;
        }
        if (ticket >= n_tickets) break;   // uniform over the workgroup
        const uint32_t combo = ticket / pixel_groups;
        const uint32_t pgroup = ticket - combo * pixel_groups;
        const int chunk = (int)(combo % (uint32_t)n_chunks);
        const int ocb = (int)(combo / (uint32_t)n_chunks);
        const int k0 = chunk * kc;
        const int kn = min(kc, p.K - k0);   // > 0: the launcher sizes n_chunks so that no chunk is empty

        if (combo != staged) {
            // stage this chunk's weights (taps k0..k0+kn-1, channels ocb*64..+63): coalesced 512 B rows
            for (int i = threadIdx.x; i < kn * 64; i += WAVES * 64)
                w_tile[i] = p.tile[(int64_t)(k0 + (i >> 6)) * p.oc_pad + ocb * 64 + (i & 63)];
            // tap table: offset of the tap inside one image relative to (iy0, ix0), and (kh, kw)
            for (int t = threadIdx.x; t < kn; t += WAVES * 64) {
                const int k = k0 + t;
                const int khw = p.KH * p.KW;
                const int ci = k / khw;
                const int r = k - ci * khw;
                const int kh = r / p.KW;
                const int kw = r - kh * p.KW;
                tap_tab[t] = make_int2((ci * p.H + kh) * p.W + kw, kh | (kw << 16));
            }
            staged = combo;
        }
        __syncthreads();

        const int oc = ocb * 64 + lane;
        // This lane's tap of the chunk (a chunk has at most 64 taps: one per lane) is the same for every pixel of
        // the ticket.  The activation of the NEXT pixel is requested before the current one is sampled, so that the
        // load's latency falls into the sampling loop.
        static_assert(kOcMaxTaps <= 64, "one tap per lane");
        const bool has_tap = lane < kn;
        const int2 info = has_tap ? tap_tab[lane] : make_int2(0, 0);
        struct Pixel { bool valid; int ox, oy, n; uint32_t pix; };
        auto locate = [&](int pp) {
            const int64_t pix = ((int64_t)pgroup * ppw + pp) * WAVES + wave;       // wave-uniform
            Pixel q;
            q.valid = pix < npix;
            const uint32_t pc = q.valid ? (uint32_t)pix : 0u;      // the number of outputs fits 32 bits
            q.pix = pc;
            const uint32_t row = pc / (uint32_t)p.OW;
            q.ox = (int)(pc - row * (uint32_t)p.OW);
            q.n = (int)(row / (uint32_t)p.OH);
            q.oy = (int)(row - (uint32_t)q.n * (uint32_t)p.OH);
            return q;
        };
        auto request = [&](const Pixel& q) {
            int32_t xv = 0;
            const int iy0 = q.oy * p.stride_h - p.pad_h, ix0 = q.ox * p.stride_w - p.pad_w;
            const int iy = iy0 + (info.y & 0xFFFF), ix = ix0 + (info.y >> 16);
            if (q.valid && has_tap && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W)
                xv = p.x[((int64_t)q.n * p.C * p.H + iy0) * p.W + ix0 + info.x];
            return xv;
        };
        // the pixel's sample range travels with its activation (a load between two pixels would make the wave wait
        // for the next pixel's activation as well); kernels for a fixed block count have no budget maps
        auto budget = [&](const Pixel& q, int pp, int& to_raw, int& from_raw) {
            if constexpr (FIXED_NB == 0) {
                const int64_t pix = ((int64_t)pgroup * ppw + pp) * WAVES + wave;
                to_raw = (q.valid && p.budget_to) ? (int)p.budget_to[pix] : p.S;
                from_raw = (q.valid && p.budget_from) ? (int)p.budget_from[pix] : 0;
            }
        };
        Pixel next = locate(0);
        int32_t xv_next = request(next);
        int to_next = 0, from_next = 0;
        budget(next, 0, to_next, from_next);
        for (int pp = 0; pp < ppw; ++pp) {
        const Pixel me = next;
        const int32_t xv = xv_next;
        const int to_raw = to_next, from_raw = from_next;
        if (pp + 1 < ppw) {
            next = locate(pp + 1);
            xv_next = request(next);
            budget(next, pp + 1, to_next, from_next);
        }
        if (me.valid) {   // wave-uniform
            const int ox = me.ox, oy = me.oy, n = me.n;

            int to, from;
            if constexpr (FIXED_NB > 0) {
                to = min(p.S, p.s_max);
                from = 0;
            } else {
                to = min(to_raw, p.s_max);
                from = min(from_raw, to);
                to = (int)uniform_u32((uint32_t)to);
                from = (int)uniform_u32((uint32_t)from);
            }

            const uint32_t o = (uint32_t)((((int64_t)n * p.OC + oc) * p.OH + oy) * p.OW + ox);
            int32_t total = 0;

            if (to > from) {
                // keep the non-zero ones of this pixel's taps of the chunk
                int cnt = 0;
                {
                    const int t = lane;
                    const unsigned long long mask = __ballot(xv != 0);
                    const int pos = cnt + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                    if (xv != 0) list[pos] = ((uint32_t)t << 8) | ((uint32_t)xv & 0xFFu);
                    cnt += __popcll(mask);
                }
                // the list is written and read by this wave only: order the LDS accesses
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

                if (cnt > 0) {
                    const uint32_t mylist = (lane < cnt) ? list[lane] : 0u;
                    PixelHoist h;
                    uint32_t hi_a;
                    mulhilo(kMulA, o, hi_a, h.lo_a);                       // round 0: MulA * o
                    const uint32_t z1 = hi_a ^ p.layer_id ^ key.k1[0];      // state word 2 after round 0
                    uint32_t lo_b1;
                    mulhilo(kMulB, z1, h.hi_b1, lo_b1);                    // round 1: MulB * z1
                    h.y2k = lo_b1 ^ key.k0[2];

                    // generator blocks serve 4 samples (32-bit uniforms) or 16 (7-bit uniforms)
                    constexpr bool p7 = FIXED_P7;
                    constexpr int lg = p7 ? 4 : 2;
                    const int j0 = from >> lg;
                    const int nb = ((to + (1 << lg) - 1) >> lg) - j0;
                    const bool full = ((from | to) & ((1 << lg) - 1)) == 0;
                    const uint32_t kbase = (uint32_t)k0;
#define PSB_LIST(NB_, VALID_, P7_) \
    total = process_list<NB_, VALID_, P7_>(mylist, cnt, w_tile, lane, kbase, j0, nb, from, to, h, key)
                    if constexpr (FIXED_NB > 0) {
                        PSB_LIST(FIXED_NB, FIXED_VALID, FIXED_P7);
                    } else if constexpr (p7) {
                        if (full && nb == 1) PSB_LIST(1, 4, true);
                        else if (full && nb == 2) PSB_LIST(2, 4, true);
                        else if (nb == 1 && (from & 15) == 0 && ((to - from) & 3) == 0) {
                            // one block, its first whole words
                            switch ((to - from) >> 2) {
                                case 1: PSB_LIST(1, 1, true); break;
                                case 2: PSB_LIST(1, 2, true); break;
                                default: PSB_LIST(1, 3, true); break;
                            }
                        } else if (nb == 1) PSB_LIST(1, 0, true);
                        else PSB_LIST(0, 0, true);
                    } else {
                    if (full) {
                        switch (nb) {
                            case 1: PSB_LIST(1, 4, false); break;
                            case 2: PSB_LIST(2, 4, false); break;
                            case 4: PSB_LIST(4, 4, false); break;
                            case 8: PSB_LIST(8, 4, false); break;
                            default: PSB_LIST(0, 0, false); break;
                        }
                    } else if (nb == 1 && (from & 3) == 0) {
                        // one block, its first to - from samples: fewer comparisons, no range checks
                        switch (to - from) {
                            case 1: PSB_LIST(1, 1, false); break;
                            case 2: PSB_LIST(1, 2, false); break;
                            default: PSB_LIST(1, 3, false); break;
                        }
                    } else if (nb == 1) {
                        PSB_LIST(1, 0, false);
                    } else {
                        PSB_LIST(0, 0, false);
                    }
                    }
#undef PSB_LIST
                }
            }

            if (oc < p.OC) {
                if (n_chunks == 1) {
                    if (p.budget_from) total += p.acc[o];
                    if (p.acc) p.acc[o] = total;
                    emit(p, o, oc, total, to);
                } else if (total != 0) {
                    // the 64 channels of the wave are 64 consecutive words: the adds of a wave are one or two
                    // requests of whole lines (in [N][OC][OH][OW] order they would be 64 lines, one plane apart,
                    // which the memory side takes 16 times more slowly)
                    atomicAdd(&p.acc_cl[(int64_t)me.pix * p.oc_pad + oc], total);
                }
            }
        }
        }   // pixels of this wave in the ticket
        // all waves are done with the tile, the lists and s_ticket before the next ticket is drawn
        __syncthreads();
    }

}

// acc[i] = 0 and, if given, the ticket counter of the persistent kernel = 0  (a plain store kernel: safe inside a
// captured graph, unlike a memset node)
__global__ void __launch_bounds__(256) k_fill_zero(int32_t* __restrict__ acc, int64_t n, uint32_t* __restrict__ sched = nullptr)
{
    if (sched && blockIdx.x == 0 && threadIdx.x == 0) sched[0] = 0u;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        acc[i] = 0;
}

// Rescaled value and/or requantised activation for layers whose accumulators were combined with atomics.
__global__ void __launch_bounds__(256) k_rescale(const LayerParams p)
{
    const int64_t total = (int64_t)p.N * p.OC * p.OH * p.OW;
    const int64_t hw = (int64_t)p.OH * p.OW;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int oc = (int)((i / hw) % p.OC);
        const int64_t pix = (i / (hw * p.OC)) * hw + (i % hw);
        int to = p.budget_to ? (int)p.budget_to[pix] : p.S;
        to = min(to, p.s_max);
        int32_t v;
        if (p.acc_cl) {     // partial sums of the channel-lane kernel, channels last (small layers: see below)
            v = p.acc_cl[pix * p.oc_pad + oc];
            if (p.budget_from) v += p.acc[i];
            if (p.acc) p.acc[i] = v;
        } else {
            v = p.acc[i];
        }
        emit(p, i, oc, v, to);
    }
}

// The same for the channel-lane kernel's split reduction, whose partial sums met in acc_cl [N*OH*OW][oc_pad]:
// acc (if given; with budget_from it holds the earlier samples' sums and the new ones are added), rescaled value
// and/or requantised activation, all [N][OC][OH][OW].  A workgroup moves a tile of 64 pixels x 64 channels through
// LDS, so that it reads whole rows of channels and writes runs of 64 pixels.  (Layers whose partial sums fit the L2
// several times over take k_rescale instead: one output per thread, more workgroups.)
__global__ void __launch_bounds__(256) k_rescale_channels_last(const LayerParams p)
{
    __shared__ int32_t tile[64][65];
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    const int64_t pix0 = (int64_t)blockIdx.x * 64;
    const int oc0 = blockIdx.y * 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll 4
    for (int r = 0; r < 16; ++r) {
        const int px = r * 4 + wave;
        tile[lane][px] = (pix0 + px < npix) ? p.acc_cl[(pix0 + px) * p.oc_pad + oc0 + lane] : 0;
    }
    __syncthreads();
    const int64_t pix = pix0 + lane;
    if (pix >= npix) return;
    const int64_t hw = (int64_t)p.OH * p.OW;
    const int64_t n = pix / hw, rem = pix - n * hw;
    int to = p.budget_to ? (int)p.budget_to[pix] : p.S;
    to = min(to, p.s_max);
#pragma unroll 4
    for (int r = 0; r < 16; ++r) {
        const int oc = oc0 + r * 4 + wave;
        if (oc >= p.OC) break;
        const int64_t o = (n * p.OC + oc) * hw + rem;
        int32_t v = tile[r * 4 + wave][lane];
        if (p.budget_from) v += p.acc[o];
        if (p.acc) p.acc[o] = v;
        emit(p, o, oc, v, to);
    }
}

// The channel-lane kernel needs groups = 1 and products that fit the 24-bit multiplier
// (|x * count| < 2^17, unit <= 2^22).
inline bool oc_lane_supported(const LayerParams& p) { return p.Cg == p.C && p.max_shift <= 22; }

inline bool oc_lane_preferred(const LayerParams& p)
{
    // at least half of the 64 lanes of the last channel block must be real channels
    return oc_lane_supported(p) && (p.OC % 64 == 0 || p.OC % 64 >= 32 || p.OC >= 256);
}

// Returns 0 or a hipError_t.
typedef bool (*ProfileBegin)(hipStream_t, int*);
typedef void (*ProfileEnd)(hipStream_t, int);

// benchmark overrides, read once per process (results do not depend on them)
struct OcTuning { int max_taps = kOcMaxTaps, ppw = 0; };
inline const OcTuning& oc_tuning()
{
    static const OcTuning tuning = [] {
        OcTuning t;
        if (const char* v = std::getenv("PSB_OC_TAPS")) { const int n = std::atoi(v); if (n >= 1 && n <= kOcMaxTaps) t.max_taps = n; }
        if (const char* v = std::getenv("PSB_OC_PPW")) { const int n = std::atoi(v); if (n >= 1 && n <= 64) t.ppw = n; }
        return t;
    }();
    return tuning;
}

inline int oc_lane_cus()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cus = n;
    }
    return cus;
}

// resident workgroups per CU: 160 KB of LDS hold four tiles; 512 VGPRs per lane hold four waves per SIMD
constexpr int kOcWgPerCu = 4;

// How the launcher cuts the tap reduction of a layer: n_chunks chunks of kc taps (at most kOcMaxTaps), as equal as
// possible, none empty; a layer too small to give every resident workgroup a ticket gets shorter chunks (down to 16
// taps) instead of leaving part of the chip idle.  With more than one chunk the partial sums meet in
// LayerParams::acc_cl, which the caller provides.
struct OcChunks { int n_chunks, kc; };
inline OcChunks oc_lane_chunks(const LayerParams& p)
{
    int max_taps = oc_tuning().max_taps;
    const int64_t n_ocb = p.oc_pad / 64;
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    const int64_t pixel_groups = (npix + kOcWaves - 1) / kOcWaves;
    OcChunks c;
    for (;;) {
        c.n_chunks = (p.K + max_taps - 1) / max_taps;
        c.kc = (p.K + c.n_chunks - 1) / c.n_chunks;
        c.n_chunks = (p.K + c.kc - 1) / c.kc;
        if (pixel_groups * c.n_chunks * n_ocb >= (int64_t)oc_lane_cus() * kOcWgPerCu || max_taps <= 16) break;
        max_taps /= 2;
    }
    return c;
}

inline int launch_oc_lane(const LayerParams& p, uint32_t* sched, hipStream_t stream, ProfileBegin prof_begin,
                          ProfileEnd prof_end)
{
    if (!oc_lane_supported(p)) return (int)hipErrorInvalidValue;
    const OcTuning& tuning = oc_tuning();
    constexpr int waves = kOcWaves;
    const int cus = oc_lane_cus();
    const int wg_per_cu = kOcWgPerCu;
    // one S everywhere, a whole number of generator blocks for which a specialised kernel is built (0: none)
    const bool p7 = p.prob_bits <= 7;
    const int per_block = p7 ? 16 : 4;
    int fixed_nb = 0, fixed_valid = 4;
    if (!p.budget_to && !p.budget_from && p.S % per_block == 0) {
        const int nb = p.S / per_block;
        if (p7 ? (nb == 1 || nb == 2) : (nb == 1 || nb == 2 || nb == 4 || nb == 8)) fixed_nb = nb;
    } else if (!p.budget_to && !p.budget_from && p7 && p.S < 16 && p.S % 4 == 0) {
        fixed_nb = 1;                       // part of one block of sixteen 7-bit uniforms: S / 4 whole words
        fixed_valid = p.S / 4;
    }
    const int n_ocb = p.oc_pad / 64;
    const int64_t npix = (int64_t)p.N * p.OH * p.OW;
    int64_t pixel_groups = (npix + waves - 1) / waves;
    const OcChunks chunks = oc_lane_chunks(p);
    const int n_chunks = chunks.n_chunks, kc = chunks.kc;
    if (n_chunks > 1 && !p.acc_cl) return (int)hipErrorInvalidValue;
    // Pixels per wave and ticket.  A ticket costs a draw, a restaging on small layers, three barriers and one
    // exposed activation load whatever it holds, so a ticket should hold some 10 us of sampling per wave (estimated
    // at half of the chunk's taps per pixel and 86 ns per generator call), which products of one or two calls only
    // reach with several pixels; large layers take four in any case (config 4: 0.66 -> 0.69 of the roofline;
    // 8 and 16 measured like 4).  Never so many that a resident workgroup would draw fewer than 1.5 tickets on
    // average (config 2 with its 7 tickets per workgroup and 11 us per ticket keeps one pixel: two measured -4 %;
    // with 7-bit uniforms, a quarter of the calls, it takes four: +16 %).
    int ppw = 1;
    {
        const double per_wg = (double)(pixel_groups * n_chunks * n_ocb) / ((double)cus * wg_per_cu);
        const int calls = p.budget_to ? 1 : (p.S + per_block - 1) / per_block;
        const double ticket_us = 0.5 * kc * calls * 0.086;
        const int want = (int)std::min(8.0, std::max(1.0, std::floor(11.0 / ticket_us + 0.5)));
        ppw = std::max(want, per_wg >= 128 ? 4 : per_wg >= 32 ? 2 : 1);
        while (ppw > 1 && per_wg / ppw < 1.5) --ppw;
        if (tuning.ppw > 0) ppw = tuning.ppw;
    }
    pixel_groups = (npix + (int64_t)waves * ppw - 1) / ((int64_t)waves * ppw);
    const int64_t n_tickets = pixel_groups * n_chunks * n_ocb;
    if (n_tickets >= (1ll << 32) - 65536) return (int)hipErrorInvalidValue;
    const int64_t grid = std::min<int64_t>(n_tickets, (int64_t)cus * wg_per_cu);

    // the ticket counter starts at 0; partial sums of a split reduction meet in accumulators that start at 0
    {
        const bool fill = n_chunks > 1;
        const int64_t words = npix * p.oc_pad;
        const int blocks = fill ? (int)std::min<int64_t>((words + 255) / 256, 8192) : 1;
        hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(fill ? 256 : 64), 0, stream, p.acc_cl, fill ? words : 0, sched);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return (int)e;
    }
    int slot = 0;
    const bool timed = prof_begin(stream, &slot);
#define PSB_OC_LAUNCH(WAVES_, NB_, P7_)                                                                           \
    hipLaunchKernelGGL((k_layer_oc_lane<WAVES_, NB_, P7_>), dim3((unsigned)grid), dim3(WAVES_ * 64), 0, stream, p,   \
                       n_chunks, kc, (uint32_t)pixel_groups, (uint32_t)n_tickets, sched, ppw)
    if (p7 && fixed_nb == 1 && fixed_valid < 4) {
        auto launch_valid = [&](auto valid_c) {
            hipLaunchKernelGGL((k_layer_oc_lane<4, 1, true, decltype(valid_c)::value>), dim3((unsigned)grid), dim3(4 * 64), 0, stream,
                               p, n_chunks, kc, (uint32_t)pixel_groups, (uint32_t)n_tickets, sched, ppw);
        };
        switch (fixed_valid) {
            case 1: launch_valid(std::integral_constant<int, 1>{}); break;
            case 2: launch_valid(std::integral_constant<int, 2>{}); break;
            default: launch_valid(std::integral_constant<int, 3>{}); break;
        }
    } else if (p7) {
        switch (fixed_nb) {
            case 1: PSB_OC_LAUNCH(4, 1, true); break;
            case 2: PSB_OC_LAUNCH(4, 2, true); break;
            default: PSB_OC_LAUNCH(4, 0, true); break;
        }
    } else {
        switch (fixed_nb) {
            case 1: PSB_OC_LAUNCH(4, 1, false); break;
            case 2: PSB_OC_LAUNCH(4, 2, false); break;
            case 4: PSB_OC_LAUNCH(4, 4, false); break;
            case 8: PSB_OC_LAUNCH(4, 8, false); break;
            default: PSB_OC_LAUNCH(4, 0, false); break;
        }
    }
#undef PSB_OC_LAUNCH
    if (timed) prof_end(stream, slot);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
    if (n_chunks > 1) {
        if ((npix + 63) / 64 > 2147483647ll) return (int)hipErrorInvalidValue;
        const int64_t total = npix * p.OC;
        if (total <= (1 << 20))
            hipLaunchKernelGGL(k_rescale, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL(k_rescale_channels_last, dim3((unsigned)((npix + 63) / 64), (unsigned)n_ocb), dim3(256), 0,
                               stream, p);
        e = hipGetLastError();
        if (e != hipSuccess) return (int)e;
    }
    return 0;
}

}  // namespace psb
