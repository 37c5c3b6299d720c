// C-ABI of the PSB layer library: argument validation, the weight handle, launches.
// See include/psb.h for the contract of every entry point.
#include "../../include/psb.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "psb_kernels.hip.h"
#include "psb_kernels_oc.hip.h"
#include "psb_kernels_list.hip.h"

struct psb_weights {
    psb_wshape shape;
    int32_t K;         // taps per output channel
    int32_t oc_pad;    // OC rounded up to a multiple of 64
    int32_t prob_bits, exp_bits, x_absmax, s_max;
    psb_winfo info;
    int device;
    uint32_t* packed_dev;    // [OC][K]
    uint2* tile_dev;         // [K][oc_pad] {threshold, unit}
    uint32_t* live_idx_dev;  // [OC][K]: live taps of each channel first, any order
    uint32_t* live_cnt_dev;  // [OC]
    uint32_t* sched_dev;     // ticket counter and finish counter of the persistent kernel (both 0 between calls)
};

namespace {

thread_local int tl_last_device_error = 0;
int g_mapping = 0;

// optional timing of the sampling kernels (psb_profile_enable / psb_profile_read)
constexpr int kMaxProfilePairs = 4096;
bool g_profile_on = false;
std::vector<hipEvent_t> g_profile_events;   // start/stop pairs, created on demand
int g_profile_used = 0;                     // pairs recorded since the last read

bool profile_begin(hipStream_t stream, int* slot)
{
    if (!g_profile_on || g_profile_used >= kMaxProfilePairs) return false;
    while ((int)g_profile_events.size() < 2 * (g_profile_used + 1)) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return false;
        g_profile_events.push_back(e);
    }
    *slot = g_profile_used;
    return hipEventRecord(g_profile_events[2 * *slot], stream) == hipSuccess;
}

void profile_end(hipStream_t stream, int slot)
{
    if (hipEventRecord(g_profile_events[2 * slot + 1], stream) == hipSuccess) g_profile_used = slot + 1;
}

#define PSB_HIP_TRY(expr)                                 \
    do {                                                  \
        hipError_t err_ = (expr);                         \
        if (err_ != hipSuccess) {                         \
            tl_last_device_error = (int)err_;             \
            return PSB_ERR_DEVICE;                        \
        }                                                 \
    } while (0)

int check_wshape(const psb_wshape* s, int64_t* K_out)
{
    if (!s) return PSB_ERR_NULL;
    if (s->oc <= 0 || s->cin <= 0 || s->kh <= 0 || s->kw <= 0 || s->groups <= 0) return PSB_ERR_SHAPE;
    if (s->cin % s->groups || s->oc % s->groups) return PSB_ERR_SHAPE;
    const int64_t K = (int64_t)(s->cin / s->groups) * s->kh * s->kw;
    if (K >= (1ll << 24)) return PSB_ERR_TOO_LARGE;   // taps are packed into 24 bits by the kernels
    if ((int64_t)s->oc * K >= (1ll << 31)) return PSB_ERR_TOO_LARGE;
    if (K_out) *K_out = K;
    return PSB_OK;
}

int check_geom(const psb_wshape* s, const psb_conv_geom* g, int32_t* oh, int32_t* ow)
{
    int rc = check_wshape(s, nullptr);
    if (rc != PSB_OK) return rc;
    if (!g) return PSB_ERR_NULL;
    if (g->n <= 0 || g->h <= 0 || g->w <= 0 || g->stride_h <= 0 || g->stride_w <= 0 || g->pad_h < 0 ||
        g->pad_w < 0)
        return PSB_ERR_SHAPE;
    if ((int64_t)g->h + 2ll * g->pad_h < s->kh || (int64_t)g->w + 2ll * g->pad_w < s->kw) return PSB_ERR_SHAPE;
    const int64_t OH = ((int64_t)g->h + 2ll * g->pad_h - s->kh) / g->stride_h + 1;
    const int64_t OW = ((int64_t)g->w + 2ll * g->pad_w - s->kw) / g->stride_w + 1;
    if ((int64_t)g->n * s->oc * OH * OW >= (1ll << 32)) return PSB_ERR_TOO_LARGE;   // counter word 0
    if ((int64_t)g->n * s->cin * g->h * g->w >= (1ll << 31)) return PSB_ERR_TOO_LARGE;
    if ((int64_t)g->pad_h >= (1 << 20) || (int64_t)g->pad_w >= (1 << 20)) return PSB_ERR_TOO_LARGE;
    if (oh) *oh = (int32_t)OH;
    if (ow) *ow = (int32_t)OW;
    return PSB_OK;
}

// Smallest admissible e_min given the per-channel exponent histogram (bin b = e_top - b).
// Returns false when even a window of one exponent can overflow.
bool choose_window(const std::vector<uint32_t>& hist, int OC, int window, int x_absmax, int s_max, int* depth)
{
    typedef unsigned __int128 u128;
    const u128 limit = (u128)2147483647u;
    for (int d = window; d >= 0; --d) {          // e_min = e_top - d, deepest window first
        u128 worst = 0;
        for (int oc = 0; oc < OC; ++oc) {
            u128 sum = 0;
            for (int b = 0; b <= d; ++b)          // exponent e_top - b, shift d - b, worst term 2^(d-b+1)
                sum += (u128)hist[(size_t)oc * psb::kHistBins + b] << (d - b + 1);
            if (sum > worst) worst = sum;
        }
        if (worst * (u128)x_absmax * (u128)s_max <= limit) { *depth = d; return true; }
    }
    return false;
}

// Which kernel serves this layer under the current mapping switch (1, 2, 3), or a psb_status.
int pick_mapping(const psb_weights* q, const psb::LayerParams& p)
{
    int mapping = g_mapping;
    if (mapping == 2 && q->shape.groups != 1) return PSB_ERR_SHAPE;
    if (mapping == 0) {
        // channel lanes pay for every (tap, channel) pair of a tile, live or not: only for mostly dense layers
        const int64_t n_weights = (int64_t)q->shape.oc * q->K;
        const bool dense = 2 * q->info.n_live >= n_weights;
        mapping = (dense && psb::oc_lane_preferred(p)) ? 2 : 3;
    }
    return mapping;
}

void fill_geometry(const psb_weights* q, const psb_conv_geom* g, int32_t OH, int32_t OW, psb::LayerParams& p)
{
    std::memset(&p, 0, sizeof(p));
    p.N = g->n; p.C = q->shape.cin; p.H = g->h; p.W = g->w;
    p.OC = q->shape.oc; p.OH = OH; p.OW = OW; p.KH = q->shape.kh; p.KW = q->shape.kw;
    p.Cg = q->shape.cin / q->shape.groups; p.OCg = q->shape.oc / q->shape.groups;
    p.K = q->K; p.oc_pad = q->oc_pad;
    p.stride_h = g->stride_h; p.stride_w = g->stride_w; p.pad_h = g->pad_h; p.pad_w = g->pad_w;
    p.s_max = q->s_max; p.prob_bits = q->prob_bits;
    p.default_mult = std::ldexp(1.0f, q->info.e_min);
    p.max_shift = q->info.e_top - q->info.e_min;
}

int launch_layer(const psb_weights* q, const int8_t* x, const psb_conv_geom* g, int32_t S,
                 const uint8_t* budget_to, const uint8_t* budget_from, uint64_t seed, uint32_t layer_id,
                 int32_t* acc, float* y, const float* mult, const float* bias, hipStream_t stream)
{
    int32_t OH = 0, OW = 0;
    int rc = check_geom(&q->shape, g, &OH, &OW);
    if (rc != PSB_OK) return rc;

    psb::LayerParams p;
    fill_geometry(q, g, OH, OW, p);
    p.packed = q->packed_dev; p.tile = q->tile_dev; p.x = x;
    p.budget_to = budget_to; p.budget_from = budget_from;
    p.acc = acc; p.y = y; p.mult = mult; p.bias = bias;
    p.S = S;
    p.key0 = (uint32_t)(seed & 0xFFFFFFFFull); p.key1 = (uint32_t)(seed >> 32); p.layer_id = layer_id;

    int dev = 0;
    PSB_HIP_TRY(hipGetDevice(&dev));
    if (dev != q->device) return PSB_ERR_DEVICE;

    const int mapping = pick_mapping(q, p);
    if (mapping < 0) return mapping;

    if (mapping == 2) {
        rc = psb::launch_oc_lane(p, q->sched_dev, stream, profile_begin, profile_end);
        if (rc != 0) { tl_last_device_error = rc; return PSB_ERR_DEVICE; }
    } else if (mapping == 3) {
        rc = psb::launch_product_list(p, q->live_idx_dev, q->live_cnt_dev, stream, profile_begin, profile_end);
        if (rc != 0) { tl_last_device_error = rc; return PSB_ERR_DEVICE; }
    } else {
        const int64_t npix = (int64_t)p.N * OH * OW;
        dim3 grid((unsigned)((npix + 255) / 256), (unsigned)p.OC, 1);
        if (p.OC > 65535) return PSB_ERR_TOO_LARGE;
        int slot = 0;
        const bool timed = profile_begin(stream, &slot);
        hipLaunchKernelGGL(psb::k_layer_pixel_lane, grid, dim3(256), 0, stream, p);
        if (timed) profile_end(stream, slot);
        PSB_HIP_TRY(hipGetLastError());
    }
    return PSB_OK;
}

}  // namespace

extern "C" {

int psb_last_device_error(void) { return tl_last_device_error; }

int psb_set_mapping(int mapping)
{
    const int prev = g_mapping;
    if (mapping >= 0 && mapping <= 3) g_mapping = mapping;
    return prev;
}

int psb_query_mapping(const psb_weights_t* q, const psb_conv_geom* geom)
{
    if (!q || !geom) return PSB_ERR_NULL;
    int32_t OH = 0, OW = 0;
    const int rc = check_geom(&q->shape, geom, &OH, &OW);
    if (rc != PSB_OK) return rc;
    psb::LayerParams p;
    fill_geometry(q, geom, OH, OW, p);
    return pick_mapping(q, p);
}

int psb_profile_enable(int on)
{
    g_profile_on = on != 0;
    if (!g_profile_on) g_profile_used = 0;
    return PSB_OK;
}

int psb_profile_read(double* kernel_ms_sum, int64_t* n_launches)
{
    if (!kernel_ms_sum || !n_launches) return PSB_ERR_NULL;
    double sum = 0.0;
    for (int i = 0; i < g_profile_used; ++i) {
        float ms = 0.0f;
        PSB_HIP_TRY(hipEventSynchronize(g_profile_events[2 * i + 1]));
        PSB_HIP_TRY(hipEventElapsedTime(&ms, g_profile_events[2 * i], g_profile_events[2 * i + 1]));
        sum += ms;
    }
    *kernel_ms_sum = sum;
    *n_launches = g_profile_used;
    g_profile_used = 0;
    return PSB_OK;
}

int psb_conv2d_out_dims(const psb_wshape* shape, const psb_conv_geom* geom, int32_t* oh, int32_t* ow)
{
    if (!shape || !geom) return PSB_ERR_NULL;
    return check_geom(shape, geom, oh, ow);
}

int psb_quantize_weights(const float* w_dev, const psb_wshape* shape, int32_t prob_bits, int32_t exp_bits,
                         int32_t x_absmax, int32_t s_max, void* hip_stream, psb_weights_t** out)
{
    if (!w_dev || !shape || !out) return PSB_ERR_NULL;
    *out = nullptr;
    int64_t K = 0;
    int rc = check_wshape(shape, &K);
    if (rc != PSB_OK) return rc;
    if (prob_bits != 23 && (prob_bits < 1 || prob_bits > 7)) return PSB_ERR_VALUE;
    if (exp_bits <= 0) exp_bits = 4;
    if (exp_bits > 5 || x_absmax <= 0 || x_absmax > 128 || s_max <= 0 || s_max > 255) return PSB_ERR_VALUE;

    hipStream_t stream = (hipStream_t)hip_stream;
    const int OC = shape->oc;
    const int oc_pad = (OC + 63) / 64 * 64;
    const int64_t nw = (int64_t)OC * K;
    const uint32_t* w_bits = reinterpret_cast<const uint32_t*>(w_dev);

    psb_weights* q = new (std::nothrow) psb_weights;
    if (!q) return PSB_ERR_ALLOC;
    std::memset(q, 0, sizeof(*q));
    q->shape = *shape; q->K = (int32_t)K; q->oc_pad = oc_pad;
    q->prob_bits = prob_bits; q->exp_bits = exp_bits; q->x_absmax = x_absmax; q->s_max = s_max;

    // scratch: [0]=max field, [1]=non-finite flag, then 3 64-bit counters, then the histogram
    uint32_t* scratch = nullptr;
    const size_t scratch_words = 8 + (size_t)OC * psb::kHistBins;
    auto fail = [&](int code, hipError_t e) {
        if (e != hipSuccess) tl_last_device_error = (int)e;
        if (scratch) (void)hipFree(scratch);
        psb_weights_destroy(q);
        return code;
    };
#define QTRY(expr)                                                   \
    do {                                                             \
        hipError_t e_ = (expr);                                      \
        if (e_ != hipSuccess) return fail(PSB_ERR_DEVICE, e_);       \
    } while (0)

    QTRY(hipGetDevice(&q->device));
    if (hipMalloc(&scratch, scratch_words * sizeof(uint32_t)) != hipSuccess) return fail(PSB_ERR_ALLOC, hipSuccess);
    if (hipMalloc(&q->packed_dev, (size_t)nw * sizeof(uint32_t)) != hipSuccess) return fail(PSB_ERR_ALLOC, hipSuccess);
    if (hipMalloc(&q->tile_dev, (size_t)oc_pad * K * sizeof(uint2)) != hipSuccess)
        return fail(PSB_ERR_ALLOC, hipSuccess);
    if (hipMalloc(&q->sched_dev, 2 * sizeof(uint32_t)) != hipSuccess) return fail(PSB_ERR_ALLOC, hipSuccess);
    if (hipMalloc(&q->live_idx_dev, (size_t)nw * sizeof(uint32_t)) != hipSuccess) return fail(PSB_ERR_ALLOC, hipSuccess);
    if (hipMalloc(&q->live_cnt_dev, (size_t)OC * sizeof(uint32_t)) != hipSuccess) return fail(PSB_ERR_ALLOC, hipSuccess);
    QTRY(hipMemsetAsync(scratch, 0, scratch_words * sizeof(uint32_t), stream));
    QTRY(hipMemsetAsync(q->sched_dev, 0, 2 * sizeof(uint32_t), stream));

    // 1. largest exponent, NaN/Inf detection
    {
        const int blocks = (int)std::min<int64_t>((nw + 255) / 256, 2048);
        hipLaunchKernelGGL(psb::k_exponent_scan, dim3(blocks), dim3(256), 0, stream, w_bits, nw, (int)prob_bits, scratch);
        QTRY(hipGetLastError());
    }
    uint32_t scan[2] = {0, 0};
    QTRY(hipMemcpyAsync(scan, scratch, sizeof(scan), hipMemcpyDeviceToHost, stream));
    QTRY(hipStreamSynchronize(stream));
    if (scan[1]) return fail(PSB_ERR_VALUE, hipSuccess);

    const int window = (1 << exp_bits) - 1;
    int field_top = (int)scan[0];
    int field_min = field_top;
    if (field_top != 0) {
        // 2. per-channel exponent histogram over the window, then the host picks e_min
        hipLaunchKernelGGL(psb::k_exponent_hist, dim3(OC), dim3(256), 0, stream, w_bits, (int)K, (int)prob_bits, field_top, window,
                           scratch + 8);
        QTRY(hipGetLastError());
        std::vector<uint32_t> hist((size_t)OC * psb::kHistBins);
        QTRY(hipMemcpyAsync(hist.data(), scratch + 8, hist.size() * sizeof(uint32_t), hipMemcpyDeviceToHost, stream));
        QTRY(hipStreamSynchronize(stream));
        int depth = 0;
        if (!choose_window(hist, OC, window, x_absmax, s_max, &depth)) return fail(PSB_ERR_OVERFLOW_UNSAFE, hipSuccess);
        field_min = field_top - depth;
        q->info.e_top = field_top - 127;
        q->info.e_min = field_min - 127;
    } else {
        q->info.e_top = 0;
        q->info.e_min = 0;
        field_min = 127;
    }
    // 3. pack
    {
        const int64_t total = (int64_t)oc_pad * K;
        const int blocks = (int)std::min<int64_t>((total + 255) / 256, 4096);
        hipLaunchKernelGGL(psb::k_pack, dim3(blocks), dim3(256), 0, stream, w_bits, OC, (int)K, oc_pad, (int)prob_bits,
                           field_min,
                           q->packed_dev, q->tile_dev, reinterpret_cast<unsigned long long*>(scratch + 2));
        QTRY(hipGetLastError());
        hipLaunchKernelGGL(psb::k_live_index, dim3(OC), dim3(256), 0, stream, q->packed_dev, (int)K, q->live_idx_dev,
                           q->live_cnt_dev);
        QTRY(hipGetLastError());
    }
    unsigned long long counts[3] = {0, 0, 0};
    QTRY(hipMemcpyAsync(counts, scratch + 2, sizeof(counts), hipMemcpyDeviceToHost, stream));
    QTRY(hipStreamSynchronize(stream));
    q->info.n_zero = (int64_t)counts[0];
    q->info.n_flushed = (int64_t)counts[1];
    q->info.n_live = (int64_t)counts[2];
    (void)hipFree(scratch);
#undef QTRY
    *out = q;
    return PSB_OK;
}

int psb_weights_info(const psb_weights_t* q, psb_winfo* info)
{
    if (!q || !info) return PSB_ERR_NULL;
    *info = q->info;
    return PSB_OK;
}

int psb_weights_export(const psb_weights_t* q, uint32_t* packed_host)
{
    if (!q || !packed_host) return PSB_ERR_NULL;
    PSB_HIP_TRY(hipMemcpy(packed_host, q->packed_dev, (size_t)q->shape.oc * q->K * sizeof(uint32_t),
                          hipMemcpyDeviceToHost));
    return PSB_OK;
}

void psb_weights_destroy(psb_weights_t* q)
{
    if (!q) return;
    if (q->packed_dev) (void)hipFree(q->packed_dev);
    if (q->tile_dev) (void)hipFree(q->tile_dev);
    if (q->sched_dev) (void)hipFree(q->sched_dev);
    if (q->live_idx_dev) (void)hipFree(q->live_idx_dev);
    if (q->live_cnt_dev) (void)hipFree(q->live_cnt_dev);
    delete q;
}

int psb_linear(const psb_weights_t* q, const int8_t* x_dev, int32_t B, int32_t S, uint64_t seed, uint32_t layer_id,
               int32_t* acc_dev, float* y_dev, const float* mult_dev, const float* bias_dev, void* hip_stream)
{
    if (!q || !x_dev || !acc_dev) return PSB_ERR_NULL;
    if (q->shape.kh != 1 || q->shape.kw != 1 || q->shape.groups != 1) return PSB_ERR_SHAPE;
    if (B <= 0) return PSB_ERR_SHAPE;
    if (S <= 0 || S > q->s_max) return PSB_ERR_VALUE;
    psb_conv_geom g = {B, 1, 1, 1, 1, 0, 0};
    return launch_layer(q, x_dev, &g, S, nullptr, nullptr, seed, layer_id, acc_dev, y_dev, mult_dev, bias_dev,
                        (hipStream_t)hip_stream);
}

int psb_conv2d(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom, int32_t S, uint64_t seed,
               uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev, const float* bias_dev,
               void* hip_stream)
{
    if (!q || !x_dev || !geom || !acc_dev) return PSB_ERR_NULL;
    if (S <= 0 || S > q->s_max) return PSB_ERR_VALUE;
    return launch_layer(q, x_dev, geom, S, nullptr, nullptr, seed, layer_id, acc_dev, y_dev, mult_dev, bias_dev,
                        (hipStream_t)hip_stream);
}

int psb_conv2d_progressive(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom,
                           const uint8_t* budget_to_dev, const uint8_t* budget_from_dev, uint64_t seed,
                           uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev,
                           const float* bias_dev, void* hip_stream)
{
    if (!q || !x_dev || !geom || !budget_to_dev || !acc_dev) return PSB_ERR_NULL;
    return launch_layer(q, x_dev, geom, 0, budget_to_dev, budget_from_dev, seed, layer_id, acc_dev, y_dev, mult_dev,
                        bias_dev, (hipStream_t)hip_stream);
}

}  // extern "C"
