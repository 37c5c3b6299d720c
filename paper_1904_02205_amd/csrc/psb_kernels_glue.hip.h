// Glue between the layers of a network (suppl. "ReLU, Batch-Norm, and Pooling": ReLU is a gate on the sign,
// max-pooling needs comparators, the factor of an average pooling is a fixed multiplication; suppl.
// "Activations and Accumulation": activations are stored as fixed-point integers).  All of these are
// streaming kernels bound by HBM bandwidth.  Every floating-point step is one binary32 operation rounded
// to nearest even (__f*_rn intrinsics: no contraction, no reassociation), in a fixed order, so that the
// integers that come out do not depend on the compiler.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "psb_kernels.hip.h"

namespace psb {

// Four elements per thread when every pointer is 16-byte (int8: 4-byte) aligned, else one.
template <bool VEC>
__global__ void __launch_bounds__(256) k_requantize(const float* __restrict__ y, const float* __restrict__ res_f32,
                                                    const int8_t* __restrict__ res_i8, float res_step, int relu,
                                                    float inv_step, float lo, float hi, int64_t n,
                                                    int8_t* __restrict__ out)
{
    const bool has_res = res_f32 || res_i8;
    if (VEC) {
        const int64_t n4 = n >> 2;
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) {
            const float4 v = reinterpret_cast<const float4*>(y)[i];
            float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
            if (res_f32) r = reinterpret_cast<const float4*>(res_f32)[i];
            if (res_i8) {
                const uint32_t b = reinterpret_cast<const uint32_t*>(res_i8)[i];
                r.x = __fmul_rn((float)(int8_t)(b & 0xFFu), res_step);
                r.y = __fmul_rn((float)(int8_t)((b >> 8) & 0xFFu), res_step);
                r.z = __fmul_rn((float)(int8_t)((b >> 16) & 0xFFu), res_step);
                r.w = __fmul_rn((float)(int8_t)(b >> 24), res_step);
            }
            const uint32_t q0 = (uint32_t)requantize_one(v.x, has_res, r.x, relu, inv_step, lo, hi) & 0xFFu;
            const uint32_t q1 = (uint32_t)requantize_one(v.y, has_res, r.y, relu, inv_step, lo, hi) & 0xFFu;
            const uint32_t q2 = (uint32_t)requantize_one(v.z, has_res, r.z, relu, inv_step, lo, hi) & 0xFFu;
            const uint32_t q3 = (uint32_t)requantize_one(v.w, has_res, r.w, relu, inv_step, lo, hi) & 0xFFu;
            reinterpret_cast<uint32_t*>(out)[i] = q0 | (q1 << 8) | (q2 << 16) | (q3 << 24);
        }
    }
    // whole array (scalar kernel) or the last n mod 4 elements (vector kernel)
    const int64_t first = VEC ? (n & ~(int64_t)3) : 0;
    for (int64_t i = first + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        float r = 0.f;
        if (res_f32) r = res_f32[i];
        if (res_i8) r = __fmul_rn((float)res_i8[i], res_step);
        out[i] = (int8_t)requantize_one(y[i], has_res, r, relu, inv_step, lo, hi);
    }
}

// Four neighbouring outputs of one row per thread (one packed 4-byte store when the row allows it); positions in
// the padding do not take part.  out_aligned: the output pointer is 4-byte aligned.
__global__ void __launch_bounds__(256) k_maxpool_i8(const int8_t* __restrict__ x, int64_t images, int H, int W, int KH,
                                                    int KW, int stride_h, int stride_w, int pad_h, int pad_w, int OH,
                                                    int OW, int out_aligned, int8_t* __restrict__ out)
{
    const int OW4 = (OW + 3) >> 2;
    const int64_t total = images * OH * OW4;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int ox0 = (int)(i % OW4) * 4;
        const int oy = (int)((i / OW4) % OH);
        const int64_t img = i / ((int64_t)OW4 * OH);
        const int8_t* src = x + img * H * W;
        int best[4] = {-128, -128, -128, -128};
        for (int dy = 0; dy < KH; ++dy) {
            const int iy = oy * stride_h - pad_h + dy;
            if ((unsigned)iy >= (unsigned)H) continue;
            const int8_t* row = src + (int64_t)iy * W;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ix0 = (ox0 + j) * stride_w - pad_w;
                for (int dx = 0; dx < KW; ++dx) {
                    const int ix = ix0 + dx;
                    if ((unsigned)ix < (unsigned)W) best[j] = max(best[j], (int)row[ix]);     // columns past OW read nothing new
                }
            }
        }
        int8_t* dst = out + (img * OH + oy) * (int64_t)OW + ox0;
        if (out_aligned && (OW & 3) == 0) {
            *reinterpret_cast<uint32_t*>(dst) = ((uint32_t)best[0] & 0xFFu) | (((uint32_t)best[1] & 0xFFu) << 8) |
                                                (((uint32_t)best[2] & 0xFFu) << 16) | (((uint32_t)best[3] & 0xFFu) << 24);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (ox0 + j < OW) dst[j] = (int8_t)best[j];
        }
    }
}

// The pooling of a ResNet stem - 3x3 windows, stride 2, padding 1 - with W and OW multiples of 4 and 4-byte aligned
// tensors: four neighbouring outputs per thread from three 32-bit loads per input row (columns 8 ox4 - 4 .. 8 ox4 + 7;
// output j takes columns 8 ox4 + 2 j - 1 .. + 1) instead of twelve byte loads, one 32-bit store.
__global__ void __launch_bounds__(256) k_maxpool_3x3s2p1_i8(const int8_t* __restrict__ x, int64_t images, int H, int W,
                                                            int OH, int OW, int8_t* __restrict__ out)
{
    const int OW4 = OW >> 2;
    const int64_t total = images * OH * OW4;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int ox4 = (int)(i % OW4);
        const int oy = (int)((i / OW4) % OH);
        const int64_t img = i / ((int64_t)OW4 * OH);
        const int8_t* src = x + img * H * W;
        int best[4] = {-128, -128, -128, -128};
#pragma unroll
        for (int dy = 0; dy < 3; ++dy) {
            const int iy = 2 * oy - 1 + dy;
            if ((unsigned)iy >= (unsigned)H) continue;
            const uint32_t* row = reinterpret_cast<const uint32_t*>(src + (int64_t)iy * W) + 2 * ox4;
            // a column outside the image does not take part: -128 cannot raise a maximum
            const uint32_t left = ox4 > 0 ? row[-1] : 0x80808080u;
            const uint32_t d0 = row[0];
            const uint32_t d1 = 8 * ox4 + 4 < W ? row[1] : 0x80808080u;
            auto byte = [](uint32_t w, int b) { return (int)(int8_t)(w >> (8 * b)); };
            best[0] = max(best[0], max(byte(left, 3), max(byte(d0, 0), byte(d0, 1))));
            best[1] = max(best[1], max(byte(d0, 1), max(byte(d0, 2), byte(d0, 3))));
            best[2] = max(best[2], max(byte(d0, 3), max(byte(d1, 0), byte(d1, 1))));
            best[3] = max(best[3], max(byte(d1, 1), max(byte(d1, 2), byte(d1, 3))));
        }
        *reinterpret_cast<uint32_t*>(out + (img * OH + oy) * (int64_t)OW + 4 * ox4) =
            ((uint32_t)best[0] & 0xFFu) | (((uint32_t)best[1] & 0xFFu) << 8) | (((uint32_t)best[2] & 0xFFu) << 16) |
            (((uint32_t)best[3] & 0xFFu) << 24);
    }
}

// Max-pooling on the blocked channels-last layout [N][H][C/32][W][32] (in and out): one thread per output pixel and
// half block of 16 channels, a 16-byte load per window position, sixteen byte-wise maxima at once.  Bytes are
// compared as unsigned numbers after their sign bits are flipped, two at a time as the 16-bit halves of a
// register (v_pk_max_u16): even bytes in one register, odd bytes in another.  Zero is the flipped -128: positions
// in the padding do not take part.
__global__ void __launch_bounds__(256) k_maxpool_blocked_i8(const int8_t* __restrict__ x, int N, int CB, int H, int W, int KH,
                                                            int KW, int stride_h, int stride_w, int pad_h, int pad_w, int OH,
                                                            int OW, int8_t* __restrict__ out)
{
    typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
    const int64_t total = (int64_t)N * OH * CB * OW * 2;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int half = (int)(i & 1);
        int64_t r = i >> 1;
        const int ox = (int)(r % OW); r /= OW;
        const int cb = (int)(r % CB); r /= CB;
        const int oy = (int)(r % OH);
        const int64_t n = r / OH;
        u16x2 even[4], odd[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) even[d] = odd[d] = u16x2{0, 0};
        for (int dy = 0; dy < KH; ++dy) {
            const int iy = oy * stride_h - pad_h + dy;
            if ((unsigned)iy >= (unsigned)H) continue;
            const int8_t* row = x + (((n * H + iy) * CB + cb) * (int64_t)W) * 32 + 16 * half;
            for (int dx = 0; dx < KW; ++dx) {
                const int ix = ox * stride_w - pad_w + dx;
                if ((unsigned)ix >= (unsigned)W) continue;
                const uint4 v = *reinterpret_cast<const uint4*>(row + (int64_t)ix * 32);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const uint32_t f = w[d] ^ 0x80808080u;
                    const uint32_t e = __builtin_amdgcn_perm(0u, f, 0x0c020c00u);     // bytes 0 and 2, zero-extended
                    const uint32_t o = __builtin_amdgcn_perm(0u, f, 0x0c030c01u);     // bytes 1 and 3
                    even[d] = __builtin_elementwise_max(even[d], __builtin_bit_cast(u16x2, e));
                    odd[d] = __builtin_elementwise_max(odd[d], __builtin_bit_cast(u16x2, o));
                }
            }
        }
        uint32_t res[4];
#pragma unroll
        for (int d = 0; d < 4; ++d)      // byte 0, byte 1, byte 2, byte 3 = even.lo, odd.lo, even.hi, odd.hi
            res[d] = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, odd[d]), __builtin_bit_cast(uint32_t, even[d]), 0x06020400u) ^
                     0x80808080u;
        *reinterpret_cast<uint4*>(out + ((((n * OH + oy) * CB + cb) * (int64_t)OW + ox) * 32 + 16 * half)) =
            make_uint4(res[0], res[1], res[2], res[3]);
    }
}

// One wave per (n, c) image: exact int32 sum, then two rounded multiplications.
__global__ void __launch_bounds__(256) k_avgpool_requantize(const int8_t* __restrict__ x, int64_t images, int HW,
                                                            float inv_count, float scale, float lo, float hi,
                                                            int8_t* __restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int64_t img = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (img >= images) return;      // wave-uniform
    const int8_t* src = x + img * HW;
    int32_t sum = 0;
    for (int i = lane; i < HW; i += 64) sum += src[i];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) out[img] = (int8_t)round_clamp(__fmul_rn(__fmul_rn(__int2float_rn(sum), inv_count), scale), lo, hi);
}

// out[n][y][x] = in[n][floor(y*H/OH)][floor(x*W/OW)]
__global__ void __launch_bounds__(256) k_budget_resample(const uint8_t* __restrict__ in, int N, int H, int W, int OH,
                                                         int OW, uint8_t* __restrict__ out)
{
    const int64_t total = (int64_t)N * OH * OW;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int ox = (int)(i % OW);
        const int oy = (int)((i / OW) % OH);
        const int64_t n = i / ((int64_t)OW * OH);
        const int64_t sy = (int64_t)oy * H / OH, sx = (int64_t)ox * W / OW;
        out[i] = in[(n * H + sy) * W + sx];
    }
}

// Attention mask (Sect. 4.5): entropy of the softmax over the channels of the last convolutional layer,
//     h = sum_c -p_c log p_c = log Z - (sum_c e_c z_c) / Z,   z_c = a_c*step - max_c, e_c = exp(z_c), Z = sum_c e_c.
// One pixel per lane; a channel of neighbouring pixels is a run of neighbouring bytes.  Evaluated in binary64
// and rounded once to binary32: sums of hundreds of binary32 terms would lose the digits the threshold
// needs, and the work (one exp per activation of ONE layer) is negligible next to the sampling kernels.
__global__ void __launch_bounds__(256) k_channel_entropy(const int8_t* __restrict__ act, float step, int N, int C,
                                                         int64_t HW, float* __restrict__ entropy)
{
    const int64_t total = (int64_t)N * HW;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t n = i / HW, px = i - n * HW;
        const int8_t* src = act + n * C * HW + px;
        int amax = -128;
        for (int c = 0; c < C; ++c) amax = max(amax, (int)src[(int64_t)c * HW]);
        double Z = 0.0, T = 0.0;
        for (int c = 0; c < C; ++c) {
            const double z = (double)((int)src[(int64_t)c * HW] - amax) * (double)step;     // <= 0
            const double e = exp(z);
            Z += e;
            T += e * z;
        }
        entropy[i] = (float)(log(Z) - T / Z);
    }
}

// One workgroup per image: mean entropy (binary64 tree sum in a fixed order), then
// budget = hi where the entropy is strictly above the mean, else lo.
__global__ void __launch_bounds__(256) k_attention_mask(const float* __restrict__ entropy, int64_t HW, uint8_t lo,
                                                        uint8_t hi, float* __restrict__ mean_out,
                                                        uint8_t* __restrict__ budget)
{
    __shared__ double part[256];
    const float* src = entropy + (int64_t)blockIdx.x * HW;
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < HW; i += 256) s += (double)src[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
        __syncthreads();
    }
    const float mean = (float)(part[0] / (double)HW);
    if (threadIdx.x == 0 && mean_out) mean_out[blockIdx.x] = mean;
    for (int64_t i = threadIdx.x; i < HW; i += 256) budget[(int64_t)blockIdx.x * HW + i] = src[i] > mean ? hi : lo;
}

}  // namespace psb
