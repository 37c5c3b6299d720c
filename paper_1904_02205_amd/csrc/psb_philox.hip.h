// Philox4x32-10 for gfx950 wavefronts (device side of the library).
//
// The generator is the published one (Salmon, Moraes, Dror, Shaw, SC'11): ten
// rounds; each round multiplies words 0 and 2 of the 4-word state by two odd
// constants, keeps the low halves, and xors the high halves with words 1 and 3
// and the two round keys; the keys advance by two Weyl constants per round.
//
// One call yields the random bits of four samples of one product: the counter is
// (o, k, sample/4, layer) and the key is the 64-bit seed (see include/psb.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace psb {

constexpr uint32_t kMulA  = 0xD2511F53u;  // multiplies state word 0
constexpr uint32_t kMulB  = 0xCD9E8D57u;  // multiplies state word 2
constexpr uint32_t kWeyl0 = 0x9E3779B9u;
constexpr uint32_t kWeyl1 = 0xBB67AE85u;

struct u32x4 { uint32_t x, y, z, w; };

// 32x32 -> 64 bit product as (hi, lo).  Written as one 64-bit multiply so the
// compiler can use a single v_mad_u64_u32 for both halves.
__device__ __forceinline__ void mulhilo(uint32_t a, uint32_t b, uint32_t& hi, uint32_t& lo)
{
    const uint64_t p = (uint64_t)a * (uint64_t)b;
    hi = (uint32_t)(p >> 32);
    lo = (uint32_t)p;
}

// One round with round keys (k0, k1).
__device__ __forceinline__ u32x4 philox_round(u32x4 c, uint32_t k0, uint32_t k1)
{
    uint32_t hi_a, lo_a, hi_b, lo_b;
    mulhilo(kMulA, c.x, hi_a, lo_a);
    mulhilo(kMulB, c.z, hi_b, lo_b);
    u32x4 r;
    r.x = hi_b ^ c.y ^ k0;
    r.y = lo_b;
    r.z = hi_a ^ c.w ^ k1;
    r.w = lo_a;
    return r;
}

// Full generator: rounds 0..9, round r uses keys (key0 + r*Weyl0, key1 + r*Weyl1).
__device__ __forceinline__ u32x4 philox4x32_10(u32x4 ctr, uint32_t key0, uint32_t key1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r)
        ctr = philox_round(ctr, key0 + (uint32_t)r * kWeyl0, key1 + (uint32_t)r * kWeyl1);
    return ctr;
}

// Rounds `first`..9 only, for callers that have already advanced the state through
// the rounds whose inputs do not depend on the tap.
template <int FIRST>
__device__ __forceinline__ u32x4 philox_rounds_from(u32x4 c, uint32_t key0, uint32_t key1)
{
#pragma unroll
    for (int r = FIRST; r < 10; ++r)
        c = philox_round(c, key0 + (uint32_t)r * kWeyl0, key1 + (uint32_t)r * kWeyl1);
    return c;
}

}  // namespace psb
