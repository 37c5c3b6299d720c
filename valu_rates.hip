// Issue-rate micro-benchmark for the integer VALU instructions the PSB kernels are made of
// (gfx950).  For each instruction class a kernel runs eight independent dependency chains
// per lane, so a SIMD never waits on a result; every SIMD of the chip holds W waves
// (W = 1, 2, 4, 8).  The shader clock is measured in the same kernels (s_memtime ticks per
// s_memrealtime tick, the latter being a 100 MHz counter), so the table is in real cycles.
//
// Output: per class, the time a SIMD needs per wave-instruction and the same in cycles.
// These figures define the ALU roofline of bench.py.
//
// Build: hipcc --offload-arch=gfx950 -O3 -I paper_1904_02205_amd/csrc valu_rates.hip -o valu_rates ; run: ./valu_rates [--json]
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "psb_philox.hip.h"

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));              \
            return 2;                                                                 \
        }                                                                             \
    } while (0)

constexpr int kChains = 8;
constexpr int kUnroll = 8;      // operations per chain per loop iteration
constexpr int kIters = 1024;

enum Op {
    OP_XOR_E32, OP_XOR_E64, OP_ADD, OP_ADD3, OP_LSHL_ADD, OP_AND_OR, OP_XAD, OP_BFI, OP_ALIGNBIT, OP_LSHR,
    OP_MAD64, OP_MULHI, OP_MULLO, OP_MAD24, OP_MUL24, OP_MULHI24,
    OP_CMP_VCC, OP_CMP_SGPR, OP_ADDC, OP_CMP_ADDC, OP_SUB_LSHR_ADD, OP_CNDMASK,
    OP_PHILOX_ROUND, OP_MAD64_SGPR, OP_XOR_SGPR, OP_PHILOX7_COUNT, OP_PHILOX10, OP_COUNT
};
static const char* kNames[OP_COUNT] = {
    "v_xor_b32 (VOP2)", "v_xor_b32_e64 (VOP3)", "v_add_u32", "v_add3_u32", "v_lshl_add_u32", "v_and_or_b32",
    "v_xad_u32", "v_bfi_b32", "v_alignbit_b32", "v_lshrrev_b32",
    "v_mad_u64_u32", "v_mul_hi_u32", "v_mul_lo_u32", "v_mad_i32_i24", "v_mul_i32_i24", "v_mul_hi_u32_u24",
    "v_cmp_lt_u32 -> vcc", "v_cmp_lt_u32_e64 -> sgpr", "v_addc_co_u32", "v_cmp_lt_u32 + v_addc_co_u32",
    "v_sub_u32 + v_lshrrev_b32 + v_add_u32", "v_cndmask_b32",
    "philox round: 2 mad_u64_u32 + 4 xor", "v_mad_u64_u32 v, s[..], v, sgpr, 0", "v_xor_b32 v, sgpr, v",
    "compiled: 7 philox rounds + 4 compare/count (= 1/8 op)", "compiled: philox4x32-10 (= 1/8 op)"};

template <int OP>
__device__ __forceinline__ void step(uint32_t& a, uint32_t& b, uint32_t m)
{
    if constexpr (OP == OP_XOR_E32) {
        asm volatile("v_xor_b32_e32 %0, %1, %0" : "+v"(a) : "v"(m));
    } else if constexpr (OP == OP_XOR_E64) {
        asm volatile("v_xor_b32_e64 %0, %1, %0" : "+v"(a) : "v"(m));
    } else if constexpr (OP == OP_ADD) {
        asm volatile("v_add_u32_e32 %0, %1, %0" : "+v"(a) : "v"(m));
    } else if constexpr (OP == OP_ADD3) {
        asm volatile("v_add3_u32 %0, %0, %1, %2" : "+v"(a) : "v"(m), "v"(b));
    } else if constexpr (OP == OP_LSHL_ADD) {
        asm volatile("v_lshl_add_u32 %0, %0, 1, %1" : "+v"(a) : "v"(m));
    } else if constexpr (OP == OP_AND_OR) {
        asm volatile("v_and_or_b32 %0, %0, %1, %2" : "+v"(a) : "v"(m), "v"(b));
    } else if constexpr (OP == OP_XAD) {
        asm volatile("v_xad_u32 %0, %0, %1, %2" : "+v"(a) : "v"(m), "v"(b));
    } else if constexpr (OP == OP_BFI) {
        asm volatile("v_bfi_b32 %0, %1, %0, %2" : "+v"(a) : "v"(m), "v"(b));
    } else if constexpr (OP == OP_ALIGNBIT) {
        asm volatile("v_alignbit_b32 %0, %0, %1, 7" : "+v"(a) : "v"(m));
    } else if constexpr (OP == OP_LSHR) {
        asm volatile("v_lshrrev_b32_e32 %0, 1, %0\n\tv_or_b32_e32 %0, %1, %0" : "+v"(a) : "v"(m));
    } else if constexpr (OP == OP_MAD64) {
        uint64_t d;
        uint64_t c = ((uint64_t)b << 32) | a;
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, %3" : "=v"(d) : "v"(a), "v"(m), "v"(c) : "vcc");
        a = (uint32_t)d;
        b = (uint32_t)(d >> 32);
    } else if constexpr (OP == OP_MULHI) {
        asm volatile("v_mul_hi_u32 %0, %0, %1" : "+v"(a) : "v"(m));
    } else if constexpr (OP == OP_MULLO) {
        asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(a) : "v"(m));
    } else if constexpr (OP == OP_MAD24) {
        asm volatile("v_mad_i32_i24 %0, %0, %1, %2" : "+v"(a) : "v"(m), "v"(b));
    } else if constexpr (OP == OP_MUL24) {
        asm volatile("v_mul_i32_i24_e32 %0, %1, %0" : "+v"(a) : "v"(m));
    } else if constexpr (OP == OP_MULHI24) {
        asm volatile("v_mul_hi_u32_u24_e32 %0, %1, %0" : "+v"(a) : "v"(m));
    } else if constexpr (OP == OP_CMP_VCC) {
        asm volatile("v_cmp_lt_u32_e32 vcc, %0, %1" : : "v"(a), "v"(m) : "vcc");
    } else if constexpr (OP == OP_CMP_SGPR) {
        uint64_t s;
        asm volatile("v_cmp_lt_u32_e64 %0, %1, %2" : "=s"(s) : "v"(a), "v"(m));
    } else if constexpr (OP == OP_ADDC) {
        asm volatile("v_addc_co_u32_e32 %0, vcc, 0, %0, vcc" : "+v"(a) : : "vcc");
    } else if constexpr (OP == OP_CMP_ADDC) {
        asm volatile("v_cmp_lt_u32_e32 vcc, %1, %2\n\tv_addc_co_u32_e32 %0, vcc, 0, %0, vcc" : "+v"(a) : "v"(b), "v"(m) : "vcc");
    } else if constexpr (OP == OP_SUB_LSHR_ADD) {
        uint32_t t;
        asm volatile("v_sub_u32_e32 %1, %2, %3\n\tv_lshrrev_b32_e32 %1, 31, %1\n\tv_add_u32_e32 %0, %1, %0"
                     : "+v"(a), "=&v"(t) : "v"(b), "v"(m));
    } else if constexpr (OP == OP_CNDMASK) {
        asm volatile("v_cndmask_b32_e32 %0, %0, %1, vcc" : "+v"(a) : "v"(m) : "vcc");
    } else if constexpr (OP == OP_PHILOX_ROUND) {
        uint64_t pa, pb;
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, 0" : "=v"(pa) : "v"(a), "v"(m) : "vcc");
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, 0" : "=v"(pb) : "v"(b), "v"(m) : "vcc");
        uint32_t x = (uint32_t)(pb >> 32), y = (uint32_t)(pa >> 32);
        asm volatile("v_xor_b32_e32 %0, %1, %0" : "+v"(x) : "v"((uint32_t)pa));
        asm volatile("v_xor_b32_e32 %0, %1, %0" : "+v"(x) : "v"(m));
        asm volatile("v_xor_b32_e32 %0, %1, %0" : "+v"(y) : "v"((uint32_t)pb));
        asm volatile("v_xor_b32_e32 %0, %1, %0" : "+v"(y) : "v"(m));
        a = x;
        b = y;
    } else if constexpr (OP == OP_MAD64_SGPR) {
        uint64_t d;
        uint64_t carry;
        asm volatile("v_mad_u64_u32 %0, %1, %2, %3, 0" : "=v"(d), "=s"(carry) : "v"(a), "s"(m));
        a = (uint32_t)d ^ (uint32_t)(d >> 32);   // one extra xor, subtracted in the table below is not attempted
    } else if constexpr (OP == OP_XOR_SGPR) {
        asm volatile("v_xor_b32_e32 %0, %1, %0" : "+v"(a) : "s"(m));
    }
}

// One "operation" = what the layer kernel does per generator call after its hoisting:
// seven full rounds and four compare/count steps, on four independent states per lane.
template <int OP>
__device__ __forceinline__ void step4(psb::u32x4 (&c)[4], uint32_t (&n)[4], uint32_t thr, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (OP == OP_PHILOX7_COUNT) {
            c[i] = psb::philox_rounds_from<3>(c[i], k0, k1);
            n[i] += (c[i].x < thr) ? 1u : 0u;
            n[i] += (c[i].y < thr) ? 1u : 0u;
            n[i] += (c[i].z < thr) ? 1u : 0u;
            n[i] += (c[i].w < thr) ? 1u : 0u;
        } else {
            c[i] = psb::philox4x32_10(c[i], k0, k1);
        }
    }
}

template <int OP>
__global__ void __launch_bounds__(256) k_rate_compiled(uint32_t* out, uint32_t m, int iters, unsigned long long* ticks)
{
    psb::u32x4 c[4];
    uint32_t n[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        c[i] = psb::u32x4{threadIdx.x * 2654435761u + i, blockIdx.x * 40503u + i, m + i, m ^ (uint32_t)i};
        n[i] = 0;
    }
    const uint32_t thr = threadIdx.x * 0x01010101u + m;
    const unsigned long long c0 = __builtin_readcyclecounter();
    const unsigned long long w0 = wall_clock64();
    // same operation count as k_rate: kUnroll * kChains "operations" per iteration, here 1/8 call each
    for (int it = 0; it < iters * 2; ++it) step4<OP>(c, n, thr, m, m * 3u);
    const unsigned long long c1 = __builtin_readcyclecounter();
    const unsigned long long w1 = wall_clock64();
    uint32_t r = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) r ^= c[i].x ^ c[i].y ^ c[i].z ^ c[i].w ^ n[i];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = r;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = c1 - c0;
        ticks[1] = w1 - w0;
    }
}

// ticks[0..1]: shader-clock and 100 MHz counter deltas of block 0, wave 0
template <int OP>
__global__ void __launch_bounds__(256) k_rate(uint32_t* out, uint32_t m, int iters, unsigned long long* ticks)
{
    uint32_t a[kChains], b[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c) {
        a[c] = threadIdx.x * 2654435761u + c;
        b[c] = blockIdx.x * 40503u + c * 7u + 1u;
    }
    const unsigned long long c0 = __builtin_readcyclecounter();
    const unsigned long long w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
#pragma unroll
            for (int c = 0; c < kChains; ++c) step<OP>(a[c], b[c], m);
    }
    const unsigned long long c1 = __builtin_readcyclecounter();
    const unsigned long long w1 = wall_clock64();
    uint32_t r = 0;
#pragma unroll
    for (int c = 0; c < kChains; ++c) r ^= a[c] ^ b[c];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = r;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = c1 - c0;
        ticks[1] = w1 - w0;
    }
}

// One generator round (two wide multiplies, four xors on their results) on the eight chains, in three instruction
// orders: 0 = chain by chain (the "philox round" row above), 1 = the sixteen multiplies, then the 32 xors,
// 2 = the multiplies of chain c between the xors of chain c - 1.  A mixed stream issues more slowly than its
// parts, and the order moves it by some 10 %.
template <int ORDER>
__global__ void __launch_bounds__(256) k_rate_round(uint32_t* out, uint32_t m, int iters, unsigned long long* ticks)
{
    uint32_t a[kChains], b[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c) {
        a[c] = threadIdx.x * 2654435761u + c;
        b[c] = blockIdx.x * 40503u + c * 7u + 1u;
    }
    auto mul = [&](uint64_t& p, uint32_t v) { asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, 0" : "=v"(p) : "v"(v), "v"(m) : "vcc"); };
    auto x2 = [&](uint32_t& x, uint32_t y) {
        asm volatile("v_xor_b32_e32 %0, %1, %0" : "+v"(x) : "v"(y));
        asm volatile("v_xor_b32_e32 %0, %1, %0" : "+v"(x) : "v"(m));
    };
    const unsigned long long c0 = __builtin_readcyclecounter();
    const unsigned long long w0 = wall_clock64();
    for (int it = 0; it < iters * kUnroll; ++it) {
        uint64_t pa[kChains], pb[kChains];
        if constexpr (ORDER == 0) {
#pragma unroll
            for (int c = 0; c < kChains; ++c) {
                mul(pa[c], a[c]);
                mul(pb[c], b[c]);
                uint32_t x = (uint32_t)(pb[c] >> 32), y = (uint32_t)(pa[c] >> 32);
                x2(x, (uint32_t)pa[c]);
                x2(y, (uint32_t)pb[c]);
                a[c] = x;
                b[c] = y;
            }
        } else if constexpr (ORDER == 1) {
#pragma unroll
            for (int c = 0; c < kChains; ++c) {
                mul(pa[c], a[c]);
                mul(pb[c], b[c]);
            }
#pragma unroll
            for (int c = 0; c < kChains; ++c) {
                uint32_t x = (uint32_t)(pb[c] >> 32), y = (uint32_t)(pa[c] >> 32);
                x2(x, (uint32_t)pa[c]);
                x2(y, (uint32_t)pb[c]);
                a[c] = x;
                b[c] = y;
            }
        } else {
#pragma unroll
            for (int c = 0; c <= kChains; ++c) {
                const int d = c - 1;
                uint32_t x = 0, y = 0;
                if (c < kChains) mul(pa[c], a[c]);
                if (c > 0) {
                    x = (uint32_t)(pb[d] >> 32);
                    x2(x, (uint32_t)pa[d]);
                }
                if (c < kChains) mul(pb[c], b[c]);
                if (c > 0) {
                    y = (uint32_t)(pa[d] >> 32);
                    x2(y, (uint32_t)pb[d]);
                    a[d] = x;
                    b[d] = y;
                }
            }
        }
    }
    const unsigned long long c1 = __builtin_readcyclecounter();
    const unsigned long long w1 = wall_clock64();
    uint32_t r = 0;
#pragma unroll
    for (int c = 0; c < kChains; ++c) r ^= a[c] ^ b[c];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = r;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = c1 - c0;
        ticks[1] = w1 - w0;
    }
}

struct Result { double ns; double clock_ghz; };

template <int OP>
static int run(uint32_t* out, unsigned long long* ticks_dev, int blocks, int waves_per_simd, Result* res)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    auto kernel = (OP == OP_PHILOX7_COUNT || OP == OP_PHILOX10) ? k_rate_compiled<OP> : k_rate<OP>;
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, 0, out, 0x9E3779B9u, 16, ticks_dev);   // warm-up
    CHECK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int rep = 0; rep < 5; ++rep) {
        CHECK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, 0, out, 0x9E3779B9u, kIters, ticks_dev);
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms = 0;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    CHECK(hipGetLastError());
    unsigned long long ticks[2];
    CHECK(hipMemcpy(ticks, ticks_dev, sizeof(ticks), hipMemcpyDeviceToHost));
    // operations of the class issued by one SIMD: waves_per_simd waves x ops per wave
    const double per_simd = (double)kIters * kUnroll * kChains * waves_per_simd;
    res->ns = (double)best * 1e6 / per_simd;
    res->clock_ghz = ticks[1] ? (double)ticks[0] / (double)ticks[1] * 0.1 : 0.0;   // 100 MHz reference
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return 0;
}

// ns per chain-round per SIMD (same operation count as the "philox round" row)
template <int ORDER>
static int run_round(uint32_t* out, unsigned long long* ticks_dev, int blocks, int waves_per_simd, Result* res)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    hipLaunchKernelGGL(k_rate_round<ORDER>, dim3(blocks), dim3(256), 0, 0, out, 0x9E3779B9u, 16, ticks_dev);   // warm-up
    CHECK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int rep = 0; rep < 5; ++rep) {
        CHECK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(k_rate_round<ORDER>, dim3(blocks), dim3(256), 0, 0, out, 0x9E3779B9u, kIters, ticks_dev);
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms = 0;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    CHECK(hipGetLastError());
    unsigned long long ticks[2];
    CHECK(hipMemcpy(ticks, ticks_dev, sizeof(ticks), hipMemcpyDeviceToHost));
    res->ns = (double)best * 1e6 / ((double)kIters * kUnroll * kChains * waves_per_simd);
    res->clock_ghz = ticks[1] ? (double)ticks[0] / (double)ticks[1] * 0.1 : 0.0;
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return 0;
}

template <int OP>
static int run_all(uint32_t* out, unsigned long long* ticks, int simds, int waves_per_simd, std::vector<Result>& r)
{
    if (run<OP>(out, ticks, simds * waves_per_simd / 4, waves_per_simd, &r[OP])) return 2;
    if constexpr (OP + 1 < OP_COUNT) return run_all<OP + 1>(out, ticks, simds, waves_per_simd, r);
    return 0;
}

int main(int argc, char** argv)
{
    const bool json = argc > 1 && std::strcmp(argv[1], "--json") == 0;
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    const int simds = cus * 4;
    uint32_t* out = nullptr;
    unsigned long long* ticks = nullptr;
    CHECK(hipMalloc(&out, (size_t)simds * 8 * 64 * sizeof(uint32_t)));
    CHECK(hipMalloc(&ticks, 2 * sizeof(unsigned long long)));
    CHECK(hipMemset(ticks, 0, 2 * sizeof(unsigned long long)));

    const int wps[4] = {1, 2, 4, 8};
    std::vector<std::vector<Result>> all(4, std::vector<Result>(OP_COUNT));
    for (int i = 0; i < 4; ++i)
        if (run_all<0>(out, ticks, simds, wps[i], all[i])) return 2;

    static const char* kOrderNames[3] = {"round, chain by chain: M M x x x x", "round, all multiplies, then all xors",
                                         "round, multiplies of chain c between the xors of c-1"};
    Result orders[4][3];
    for (int i = 0; i < 4; ++i) {
        const int blocks = simds * wps[i] / 4;
        if (run_round<0>(out, ticks, blocks, wps[i], &orders[i][0])) return 2;
        if (run_round<1>(out, ticks, blocks, wps[i], &orders[i][1])) return 2;
        if (run_round<2>(out, ticks, blocks, wps[i], &orders[i][2])) return 2;
    }

    if (json) {
        std::printf("{\"device\": \"%s\", \"cus\": %d, \"reported_clock_mhz\": %d, \"waves_per_simd\": [1, 2, 4, 8], \"ops\": {",
                    prop.gcnArchName, cus, prop.clockRate / 1000);
        for (int op = 0; op < OP_COUNT; ++op) {
            std::printf("%s\"%s\": {\"ns\": [%.4f, %.4f, %.4f, %.4f], \"measured_clock_ghz\": %.3f}", op ? ", " : "",
                        kNames[op], all[0][op].ns, all[1][op].ns, all[2][op].ns, all[3][op].ns, all[2][op].clock_ghz);
        }
        std::printf("}, \"round_orders\": {");
        for (int o = 0; o < 3; ++o)
            std::printf("%s\"%s\": {\"ns\": [%.4f, %.4f, %.4f, %.4f], \"measured_clock_ghz\": %.3f}", o ? ", " : "",
                        kOrderNames[o], orders[0][o].ns, orders[1][o].ns, orders[2][o].ns, orders[3][o].ns, orders[2][o].clock_ghz);
        std::printf("}}\n");
    } else {
        std::printf("device %s, %d CUs, reported clock %d MHz\n", prop.gcnArchName, cus, prop.clockRate / 1000);
        std::printf("ns per wave-op per SIMD at 1/2/4/8 waves per SIMD; cycles = ns x measured shader clock (4 waves)\n");
        for (int op = 0; op < OP_COUNT; ++op)
            std::printf("%-40s %7.3f %7.3f %7.3f %7.3f   clock %.3f GHz  -> %6.2f cycles\n", kNames[op], all[0][op].ns,
                        all[1][op].ns, all[2][op].ns, all[3][op].ns, all[2][op].clock_ghz,
                        all[2][op].ns * all[2][op].clock_ghz);
        for (int o = 0; o < 3; ++o)
            std::printf("%-52s %7.3f %7.3f %7.3f %7.3f   clock %.3f GHz  -> %6.2f cycles\n", kOrderNames[o], orders[0][o].ns,
                        orders[1][o].ns, orders[2][o].ns, orders[3][o].ns, orders[2][o].clock_ghz,
                        orders[2][o].ns * orders[2][o].clock_ghz);
    }
    CHECK(hipFree(out));
    CHECK(hipFree(ticks));
    return 0;
}
