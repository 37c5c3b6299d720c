// C-ABI of the PSB layer library: argument validation, the weight handle, launches.
// See include/psb.h for the contract of every entry point.
#include "../../include/psb.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "psb_kernels.hip.h"
#include "psb_kernels_oc.hip.h"
#include "psb_kernels_list.hip.h"
#include "psb_kernels_shared.hip.h"
#include "psb_kernels_glue.hip.h"

// Device memory of the shared-filter mode; allocated on first use, grown on demand, owned by the handle.
struct shared_workspace {
    int32_t* w32_dev = nullptr;      // [OC][K] sampled integer filter
    int8_t* planes_dev = nullptr;    // digit planes in matrix-core operand order, one buffer per segment of the sample axis
    int planes_segments = 0;         // segments the allocation holds
    uint8_t* qmap_dev = nullptr;     // a budget map rounded down to announced levels (calls that cannot take them in one launch)
    size_t qmap_bytes = 0;
    int8_t* xt_dev = nullptr;        // blocked channels-last copy of the activations
    size_t xt_bytes = 0;
    uint32_t* present_dev = nullptr; // 256 flags: budget values that occur
    int32_t* acc_dev = nullptr;      // accumulators of calls that do not hand any out but combine partial sums
    size_t acc_bytes = 0;
    // digit planes sampled ahead of the call by psb_shared_prepare_filters; the next matching call consumes them
    bool ready = false;
    uint64_t ready_seed = 0;
    uint32_t ready_layer = 0;
    int ready_n_seg = 0;             // segments [0, l_1), [l_1, l_2), ... of the sample axis; a uniform S is one segment
    int ready_level[4] = {0, 0, 0, 0};
};

// Accumulator scratch of a handle for psb_conv2d_requant calls without acc_dev (grown on demand).
int32_t* scratch_acc(shared_workspace* ws, size_t bytes, hipStream_t stream)
{
    if (ws->acc_bytes < bytes) {
        if (ws->acc_dev) {
            if (hipStreamSynchronize(stream) != hipSuccess) return nullptr;   // an earlier call may still use it
            (void)hipFree(ws->acc_dev);
            ws->acc_dev = nullptr;
            ws->acc_bytes = 0;
        }
        if (hipMalloc(&ws->acc_dev, bytes) != hipSuccess) return nullptr;
        ws->acc_bytes = bytes;
    }
    return ws->acc_dev;
}

// Scratch memory of psb_conv2d_requant_static: the ticket counter of the persistent layer kernel (first word of a
// 256-byte head) and the accumulators in which the partial sums of a split tap reduction meet.  A file-scope device
// array, so that the entry point never allocates; every GPU the library runs on holds its own copy at its own
// address until the process ends.  Host code never uses the array's name as an address: the per-device pointer
// comes from hipGetSymbolAddress (static_scratch() below).
constexpr size_t kStaticHeadWords = 64;
constexpr size_t kStaticAccWords = (size_t)PSB_STATIC_MAX_OUTPUTS;
static __device__ __align__(256) uint32_t scratch[kStaticHeadWords + kStaticAccWords];

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
    shared_workspace* ws;    // shared-filter mode
};

namespace {

thread_local int tl_last_device_error = 0;
// budget values announced by psb_shared_budget_levels for the thread's next shared-filter call with a budget map
// (n = 0: none, the call reads them back from its maps)
thread_local int tl_levels_n = 0;
thread_local uint8_t tl_levels[256];
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

// Device address of `scratch` on device dev, which must be the current device.  Resolved once per device (by
// psb_quantize_weights, the set-up call of every handle, or else by the first call that needs it) and kept.
constexpr int kMaxDevices = 64;
uint32_t* g_static_scratch[kMaxDevices] = {};
std::mutex g_static_scratch_mutex;

int static_scratch(int dev, uint32_t** out)
{
    if (dev < 0 || dev >= kMaxDevices) return PSB_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch[dev]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            tl_last_device_error = (int)e;
            return PSB_ERR_DEVICE;
        }
        g_static_scratch[dev] = static_cast<uint32_t*>(ptr);
    }
    if (out) *out = g_static_scratch[dev];
    return PSB_OK;
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
    if (s->kh >= (1 << 15) || s->kw >= (1 << 15)) return PSB_ERR_TOO_LARGE;   // and a tap's (kh, kw) into two 16-bit halves
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
                 int32_t* acc, float* y, const float* mult, const float* bias, hipStream_t stream,
                 const psb::Requant* rq = nullptr, bool use_static_scratch = false)
{
    int32_t OH = 0, OW = 0;
    int rc = check_geom(&q->shape, g, &OH, &OW);
    if (rc != PSB_OK) return rc;
    // the static array holds the partial sums with the channel count rounded up to whole blocks of 64
    if (use_static_scratch && (int64_t)g->n * q->oc_pad * OH * OW > (int64_t)kStaticAccWords) return PSB_ERR_TOO_LARGE;

    psb::LayerParams p;
    fill_geometry(q, g, OH, OW, p);
    p.packed = q->packed_dev; p.tile = q->tile_dev; p.x = x;
    p.budget_to = budget_to; p.budget_from = budget_from;
    p.acc = acc; p.y = y; p.mult = mult; p.bias = bias;
    if (rq) p.rq = *rq;
    p.S = S;
    p.key0 = (uint32_t)(seed & 0xFFFFFFFFull); p.key1 = (uint32_t)(seed >> 32); p.layer_id = layer_id;

    int dev = 0;
    PSB_HIP_TRY(hipGetDevice(&dev));
    if (dev != q->device) return PSB_ERR_DEVICE;

    const int mapping = pick_mapping(q, p);
    if (mapping < 0) return mapping;
    uint32_t* sched = q->sched_dev;
    // the channel-lane kernel combines the partial sums of a split tap reduction in scratch accumulators
    const bool split = mapping == 2 && psb::oc_lane_chunks(p).n_chunks > 1;
    if (use_static_scratch) {           // ticket counter and accumulators in the static array: nothing is allocated
        uint32_t* base = nullptr;
        rc = static_scratch(dev, &base);
        if (rc != PSB_OK) return rc;
        sched = base;
        if (split) p.acc_cl = reinterpret_cast<int32_t*>(base + kStaticHeadWords);
    } else if (split) {
        p.acc_cl = scratch_acc(q->ws, (size_t)p.N * OH * OW * (size_t)p.oc_pad * sizeof(int32_t), stream);
        if (!p.acc_cl) return PSB_ERR_ALLOC;
    }

    if (mapping == 2) {
        rc = psb::launch_oc_lane(p, sched, stream, profile_begin, profile_end);
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

// ---- shared-filter mode -----------------------------------------------------------------------------

psb::FilterJob filter_job(const psb_weights* q, int from, int to, uint64_t seed, uint32_t layer_id, int32_t* w32,
                          int8_t* planes, int CB, int n_ksteps)
{
    psb::FilterJob j;
    j.packed = q->packed_dev; j.OC = q->shape.oc; j.K = q->K; j.KHW = q->shape.kh * q->shape.kw;
    j.CB = CB; j.n_ksteps = n_ksteps; j.prob_bits = q->prob_bits; j.from = from; j.to = to;
    j.key0 = (uint32_t)(seed & 0xFFFFFFFFull); j.key1 = (uint32_t)(seed >> 32); j.layer_id = layer_id;
    j.w32 = w32; j.planes = planes;
    j.pack_KW = 0; j.pack_C = 0; j.n_planes = psb::kMaxPlanes;
    j.C = q->K / j.KHW;
    j.inv_ksteps = psb::inverse_of((uint32_t)n_ksteps); j.inv_CB = psb::inverse_of((uint32_t)CB); j.inv_pack_C = 0xFFFFFFFFu;
    return j;
}

int sample_filter_launch(const psb_weights* q, int from, int to, uint64_t seed, uint32_t layer_id, int32_t* w32,
                         int8_t* planes, int CB, int n_ksteps, hipStream_t stream)
{
    const int64_t nw = (int64_t)q->shape.oc * q->K;
    hipLaunchKernelGGL(psb::k_sample_filter, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, stream,
                       filter_job(q, from, to, seed, layer_id, w32, planes, CB, n_ksteps));
    PSB_HIP_TRY(hipGetLastError());
    return PSB_OK;
}

// How a handle's shared-filter calls run: on the matrix cores or with the direct kernel, and the shape of the
// digit planes.  Depends on the weight shape (and the mapping switch) only.
struct shared_plan {
    bool mfma, rowpack;
    int C_pad, CB, n_ksteps, n_ocb;
};

shared_plan plan_shared(const psb_weights* q)
{
    shared_plan s;
    s.mfma = q->shape.groups == 1 && g_mapping != 1;
    // Layers with very few input channels (a network's first layer): pack the kw x C values of one kernel row
    // into one 32-byte reduction block instead of padding every tap's C channels to 32.
    s.rowpack = s.mfma && q->shape.kw > 1 && q->shape.kw * q->shape.cin <= 32;
    s.C_pad = s.rowpack ? 32 : (q->shape.cin + 31) / 32 * 32;
    s.CB = s.C_pad / 32;
    s.n_ksteps = s.rowpack ? q->shape.kh : q->shape.kh * q->shape.kw * s.CB;
    s.n_ocb = (q->shape.oc + 31) / 32;
    return s;
}

// Bytes of the digit planes of one segment (one chunk of padding: the kernel stages whole chunks of reduction steps).
size_t planes_segment_bytes(const shared_plan& sp)
{
    return (size_t)(sp.n_ocb * sp.n_ksteps + psb::kStageSteps) * psb::kMaxPlanes * psb::kPlaneStride;
}

// The digit-plane buffer of a handle for n_seg segments (allocated on first use, grown when a call has more
// segments than any before; growing synchronises the stream first: an earlier call may still read the old buffer).
int ensure_planes(const psb_weights* q, const shared_plan& sp, int n_seg, hipStream_t stream)
{
    // each digit plane is summed in int32: 128 * 128 * (padded reduction length) must stay below 2^31
    if ((int64_t)sp.n_ksteps * 32 * n_seg >= (1ll << 17)) return PSB_ERR_TOO_LARGE;
    shared_workspace* ws = q->ws;
    if (ws->planes_segments < n_seg) {
        if (ws->planes_dev) {
            PSB_HIP_TRY(hipStreamSynchronize(stream));
            (void)hipFree(ws->planes_dev);
            ws->planes_dev = nullptr;
            ws->planes_segments = 0;
            ws->ready = false;
        }
        if (hipMalloc(&ws->planes_dev, planes_segment_bytes(sp) * n_seg) != hipSuccess) return PSB_ERR_ALLOC;   // written whole by every sampling
        ws->planes_segments = n_seg;
    }
    return PSB_OK;
}

// Sorted distinct non-zero levels, clamped to s_max; at most 4 are taken in one launch (more: returns -1).
int normalise_levels(const uint8_t* levels, int n, int s_max, int (&out)[4])
{
    bool seen[256] = {};
    for (int i = 0; i < n; ++i) seen[std::min<int>(levels[i], s_max)] = true;
    int m = 0;
    for (int v = 1; v < 256; ++v)
        if (seen[v]) {
            if (m == 4) return -1;
            out[m++] = v;
        }
    return m;
}

// One launch that samples the digit planes of segments [0, l_1), [l_1, l_2), ... of a handle.
int sample_segments(const psb_weights* q, const shared_plan& sp, const int (&level)[4], int n_seg, uint64_t seed,
                    uint32_t layer_id, int n_planes, hipStream_t stream)
{
    psb::FilterBatch batch;
    std::memset(&batch, 0, sizeof(batch));
    for (int k = 0; k <= psb::kMaxBatchJobs; ++k) batch.first_block[k] = 0xFFFFFFFFu;
    const int64_t need = ((int64_t)sp.n_ocb * sp.n_ksteps + psb::kPlaneGroup - 1) / psb::kPlaneGroup * 4;
    if (need * n_seg > 2147483647ll) return PSB_ERR_TOO_LARGE;
    for (int i = 0; i < n_seg; ++i) {
        psb::FilterJob fj = filter_job(q, i == 0 ? 0 : level[i - 1], level[i], seed, layer_id, nullptr,
                                       q->ws->planes_dev + planes_segment_bytes(sp) * i, sp.CB, sp.n_ksteps);
        fj.n_planes = n_planes;
        if (sp.rowpack) { fj.pack_KW = q->shape.kw; fj.pack_C = q->shape.cin; fj.inv_pack_C = psb::inverse_of((uint32_t)q->shape.cin); }
        batch.jobs[i] = fj;
        batch.first_block[i] = (unsigned)(need * i);
    }
    hipLaunchKernelGGL(psb::k_sample_planes_batch, dim3((unsigned)(need * n_seg)), dim3(256), 0, stream, batch);
    PSB_HIP_TRY(hipGetLastError());
    return PSB_OK;
}

// layout: PSB_BLOCKED_IN | PSB_BLOCKED_OUT | PSB_BLOCKED_RES
int launch_shared(const psb_weights* q, const int8_t* x, const psb_conv_geom* g, int32_t S, const uint8_t* budget_to,
                  const uint8_t* budget_from, uint64_t seed, uint32_t layer_id, int32_t* acc, float* y,
                  const float* mult, const float* bias, hipStream_t stream, const psb::Requant* rq = nullptr,
                  int layout = 0, const uint8_t* levels = nullptr, int n_levels = 0)
{
    int32_t OH = 0, OW = 0;
    int rc = check_geom(&q->shape, g, &OH, &OW);
    if (rc != PSB_OK) return rc;
    int dev = 0;
    PSB_HIP_TRY(hipGetDevice(&dev));
    if (dev != q->device) return PSB_ERR_DEVICE;
    // Levels given with the call: budgets are rounded DOWN to them.  Levels announced by psb_shared_budget_levels
    // are for this call only and must cover the maps (nothing is rounded).
    const bool round_down = budget_to && levels && n_levels > 0;
    uint8_t announced[256];
    int n_announced = 0;
    if (budget_to && !round_down && tl_levels_n > 0) {
        n_announced = tl_levels_n;
        std::memcpy(announced, tl_levels, (size_t)n_announced);
    }
    if (budget_to) tl_levels_n = 0;                 // announced levels are used once
    int seg_level[4] = {0, 0, 0, 0};
    int n_seg = round_down ? normalise_levels(levels, n_levels, q->s_max, seg_level) : 0;

    const shared_plan sp = plan_shared(q);
    const bool mfma = sp.mfma, rowpack = sp.rowpack;
    const int C_pad = sp.C_pad, CB = sp.CB, n_ksteps = sp.n_ksteps, n_ocb = sp.n_ocb;
    bool in_blocked = (layout & PSB_BLOCKED_IN) != 0;
    // a blocked input is read in place by the matrix-core kernel; the other kernels have no use for it
    if (in_blocked && (!mfma || rowpack)) return PSB_ERR_SHAPE;
    if (in_blocked && ((uintptr_t)x & 15u) != 0) return PSB_ERR_VALUE;
    // a 1 x 1 image with whole channel blocks (a linear layer) has the same bytes in both layouts: no copy needed
    if (mfma && !rowpack && g->h == 1 && g->w == 1 && q->shape.cin % 32 == 0 && ((uintptr_t)x & 15u) == 0)
        in_blocked = true;

    shared_workspace* ws = q->ws;
    const int64_t nw = (int64_t)q->shape.oc * q->K;
    if (!mfma && !ws->w32_dev && hipMalloc(&ws->w32_dev, (size_t)nw * sizeof(int32_t)) != hipSuccess)
        return PSB_ERR_ALLOC;
    if (!ws->present_dev && hipMalloc(&ws->present_dev, 256 * sizeof(uint32_t)) != hipSuccess) return PSB_ERR_ALLOC;
    // ksplit and the tile shape decide whether the segments can share one launch: computed before the planes are sized
    int ksplit = 1, half_tiles = 2;
    if (mfma) {
        // Few pixel tiles and a long reduction: cut the reduction so that every SIMD has a wave.  Only then: the
        // partial sums cost a zero-fill, atomics and a separate rescale pass, which measured slower than the
        // unsplit kernel as soon as the chip is half full.
        half_tiles = psb::shared_half_tiles((int64_t)g->n * OH * OW, n_ocb);
        const int64_t waves = ((int64_t)g->n * OH * OW + 32 * half_tiles - 1) / (32 * half_tiles) * n_ocb;
        const int64_t want = waves <= 512 ? (1024 + waves - 1) / waves : 1;
        ksplit = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, 8), n_ksteps / 16));
        // the 3 x 3 kernel with both operands in LDS deals the channel blocks to teams inside a workgroup instead
        if (!rowpack && psb::window_slots(q->shape.kh, q->shape.kw, g->stride_h, g->stride_w, g->pad_h, g->pad_w, g->h, g->w,
                                          half_tiles) > 0)
            ksplit = 1;
    }
    // all segments in one launch, accumulated in registers, epilogue fused
    const bool fused_segments = round_down && mfma && n_seg > 0 && !budget_from && ksplit == 1 &&
                                (int64_t)n_ksteps * 32 * n_seg < (1ll << 17);
    if (mfma) {
        rc = ensure_planes(q, sp, fused_segments ? n_seg : 1, stream);
        if (rc != PSB_OK) return rc;
    }
    if (round_down && !fused_segments) {
        // This call takes the segments one launch at a time (direct kernel, split reduction, more than four
        // levels): round the map down to the levels first, then it is a map that holds only announced values.
        const size_t need = (size_t)g->n * OH * OW;
        if (ws->qmap_bytes < need) {
            if (ws->qmap_dev) {
                PSB_HIP_TRY(hipStreamSynchronize(stream));
                (void)hipFree(ws->qmap_dev);
                ws->qmap_dev = nullptr;
                ws->qmap_bytes = 0;
            }
            if (hipMalloc(&ws->qmap_dev, need) != hipSuccess) return PSB_ERR_ALLOC;
            ws->qmap_bytes = need;
        }
        uint8_t all[256];
        int n_all = 0;
        {
            bool seen[256] = {};
            for (int i = 0; i < n_levels; ++i) seen[std::min<int>(levels[i], q->s_max)] = true;
            for (int v = 1; v < 256; ++v) if (seen[v]) all[n_all++] = (uint8_t)v;
        }
        if (n_all <= 4) {
            psb::BudgetLevels bl;
            bl.n = n_all;
            for (int i = 0; i < 4; ++i) bl.level[i] = i < n_all ? all[i] : 0;
            const int blocks = (int)std::min<int64_t>(((int64_t)need + 255) / 256, 1024);
            hipLaunchKernelGGL(psb::k_budget_round_down, dim3(blocks), dim3(256), 0, stream, budget_to, (int64_t)need,
                               q->s_max, bl, ws->qmap_dev);
            PSB_HIP_TRY(hipGetLastError());
        } else {
            return PSB_ERR_VALUE;           // more than four levels
        }
        budget_to = ws->qmap_dev;
        n_announced = n_all;
        std::memcpy(announced, all, (size_t)n_all);
    }
    // blocked channels-last copy (row-packed: one 32-byte block per input row and output column)
    const size_t xt_need = (size_t)g->n * g->h * (rowpack ? OW : g->w) * C_pad;
    if (mfma && xt_need >= (1ull << 31)) return PSB_ERR_TOO_LARGE;      // the kernel addresses it with 32-bit offsets
    if (mfma && !in_blocked && ws->xt_bytes < xt_need) {
        if (ws->xt_dev) {
            PSB_HIP_TRY(hipStreamSynchronize(stream));     // an earlier call may still read the old buffer
            (void)hipFree(ws->xt_dev);
            ws->xt_dev = nullptr;
            ws->xt_bytes = 0;
        }
        if (hipMalloc(&ws->xt_dev, xt_need) != hipSuccess) return PSB_ERR_ALLOC;
        ws->xt_bytes = xt_need;
    }

    psb::SharedParams p;
    std::memset(&p, 0, sizeof(p));
    p.x = x; p.xt = in_blocked ? x : ws->xt_dev; p.planes = ws->planes_dev; p.w32 = ws->w32_dev;
    p.budget_to = budget_to; p.budget_from = budget_from;
    p.acc = acc; p.y = y; p.mult = mult; p.bias = bias;
    if (rq) p.rq = *rq;
    p.N = g->n; p.C = q->shape.cin; p.H = g->h; p.W = g->w;
    p.OC = q->shape.oc; p.OH = OH; p.OW = OW; p.KH = q->shape.kh; p.KW = q->shape.kw;
    p.Cg = q->shape.cin / q->shape.groups; p.OCg = q->shape.oc / q->shape.groups;
    p.K = q->K; p.C_pad = C_pad; p.n_ksteps = n_ksteps;
    p.stride_h = g->stride_h; p.stride_w = g->stride_w; p.pad_h = g->pad_h; p.pad_w = g->pad_w;
    p.S = S; p.s_max = q->s_max;
    p.default_mult = std::ldexp(1.0f, q->info.e_min);
    p.xt_bytes = (uint32_t)xt_need;
    p.tH = g->h; p.tW = g->w; p.tKH = q->shape.kh; p.tKW = q->shape.kw;
    p.t_stride_h = g->stride_h; p.t_stride_w = g->stride_w; p.t_pad_h = g->pad_h; p.t_pad_w = g->pad_w;
    if (rowpack) { p.tW = OW; p.tKW = 1; p.t_stride_w = 1; p.t_pad_w = 0; }
    p.inv_OW = psb::inverse_of((uint32_t)OW); p.inv_OH = psb::inverse_of((uint32_t)OH);
    p.inv_W1 = psb::inverse_of((uint32_t)p.tW + 1u); p.inv_H1 = psb::inverse_of((uint32_t)p.tH + 1u);
    const bool words = ((int64_t)OH * OW) % 4 == 0;
    p.quad_store = rq && rq->x_out && !rq->out_blocked && words && ((uintptr_t)rq->x_out & 3u) == 0;
    p.quad_res = rq && rq->res_i8 && !rq->res_blocked && words && ((uintptr_t)rq->res_i8 & 3u) == 0;
    if (rq && ((rq->out_blocked && ((uintptr_t)rq->x_out & 3u) != 0) ||
               (rq->res_blocked && ((uintptr_t)rq->res_i8 & 3u) != 0)))
        return PSB_ERR_VALUE;
    p.ksplit = ksplit;
    const int max_shift = q->info.e_top - q->info.e_min;
    const int64_t npix = (int64_t)g->n * OH * OW;
    if (!mfma && p.OC > 65535) return PSB_ERR_TOO_LARGE;

    // preparation: sample the filter of the first (or only) segment and, for the matrix cores, transpose the
    // activations - one launch for both
    psb::TransposeJob tj;
    std::memset(&tj, 0, sizeof(tj));
    int64_t transpose_blocks = 0;
    if (mfma && !in_blocked) {
        tj.x = x; tj.C = p.C; tj.H = p.H; tj.W = p.W; tj.C_pad = C_pad; tj.xt = ws->xt_dev;
        tj.wide = ((int64_t)g->h * g->w) % 4 == 0 && ((uintptr_t)x & 3u) == 0;
        const int per_tile = tj.wide ? psb::kWideTilePositions : 64;
        tj.N = g->n; tj.tiles_p = (int)(((int64_t)g->h * g->w + per_tile - 1) / per_tile); tj.rows = (int64_t)g->n * g->h;
        transpose_blocks = (int64_t)tj.tiles_p * g->n * CB;
        if (rowpack) {
            tj.pack_KW = q->shape.kw; tj.OW = OW; tj.stride_w = g->stride_w; tj.pad_w = g->pad_w;
            transpose_blocks = (tj.rows * OW + 255) / 256;
        }
    }
    auto prepare = [&](int from, int to) -> int {
        // matrix cores: one thread per slot of the operand-ordered planes; otherwise one per weight
        // planes sampled ahead of this call (psb_shared_prepare_filters) are used once
        const bool have = mfma && ws->ready && ws->ready_seed == seed && ws->ready_layer == layer_id && from == 0 &&
                          ws->ready_n_seg == 1 && to == ws->ready_level[0];
        ws->ready = false;
        const int64_t filter_blocks = have ? 0 : mfma ? ((int64_t)n_ocb * n_ksteps + psb::kPlaneGroup - 1) / psb::kPlaneGroup * 4 : (nw + 255) / 256;
        if (filter_blocks + transpose_blocks > 2147483647ll) return PSB_ERR_TOO_LARGE;
        if (filter_blocks + transpose_blocks == 0) return PSB_OK;
        psb::FilterJob fj = filter_job(q, from, to, seed, layer_id, mfma ? nullptr : ws->w32_dev,
                                       mfma ? ws->planes_dev : nullptr, CB, n_ksteps);
        fj.n_planes = psb::planes_needed(max_shift, to - from);
        if (rowpack) { fj.pack_KW = q->shape.kw; fj.pack_C = q->shape.cin; fj.inv_pack_C = psb::inverse_of((uint32_t)q->shape.cin); }
        hipLaunchKernelGGL(psb::k_shared_prologue, dim3((unsigned)(filter_blocks + transpose_blocks)), dim3(256), 0,
                           stream, fj, tj, (unsigned)filter_blocks);
        PSB_HIP_TRY(hipGetLastError());
        transpose_blocks = 0;                       // once per call
        return PSB_OK;
    };

    auto contract = [&](int n_samples) -> int {
        int slot = 0;
        const bool timed = profile_begin(stream, &slot);
        if (mfma) {
            static const int resident_wgs = [] {
                if (const char* v = std::getenv("PSB_SHARED_RESIDENT")) { if (std::atoi(v) == 0) return 0; }   // benchmark switch
                int dev = 0, n = 0;
                if (hipGetDevice(&dev) != hipSuccess ||
                    hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
                    n = 256;
                return 2 * n;
            }();
            psb::launch_conv_shared_mfma(p, psb::planes_needed(max_shift, n_samples), resident_wgs, half_tiles, stream);
        } else {
            const int64_t columns = (npix + 255) / 256;
            if (p.Cg == 1 && p.KH == 3 && p.KW == 3) {
                // several channels per workgroup row while that leaves eight waves for every SIMD of the chip
                int channels = 8;
                while (channels > 2 && columns * ((p.OC + channels - 1) / channels) < 2048) channels /= 2;
                const dim3 grid((unsigned)columns, (unsigned)((p.OC + channels - 1) / channels));
                hipLaunchKernelGGL((psb::k_conv_shared_depthwise<3, 3>), grid, dim3(256), 0, stream, p, channels);
            } else {
                const dim3 grid((unsigned)columns, (unsigned)p.OC);
                hipLaunchKernelGGL(psb::k_conv_shared_direct, grid, dim3(256), 0, stream, p);
            }
        }
        if (timed) profile_end(stream, slot);
        PSB_HIP_TRY(hipGetLastError());
        return PSB_OK;
    };

    const int64_t total = npix * p.OC;
    if (!acc && !fused_segments && (p.ksplit > 1 || budget_to)) {      // partial sums meet in the accumulators
        acc = scratch_acc(ws, (size_t)total * sizeof(int32_t), stream);
        if (!acc) return PSB_ERR_ALLOC;
        p.acc = acc;
    }
    auto rescale_pass = [&]() -> int {
        psb::LayerParams lp;
        fill_geometry(q, g, OH, OW, lp);
        lp.acc = acc; lp.y = y; lp.mult = mult; lp.bias = bias; lp.budget_to = budget_to; lp.S = S;
        if (rq) lp.rq = *rq;
        const int blocks = (int)std::min<int64_t>((total + 255) / 256, 8192);
        hipLaunchKernelGGL(psb::k_rescale, dim3(blocks), dim3(256), 0, stream, lp);
        PSB_HIP_TRY(hipGetLastError());
        return PSB_OK;
    };
    auto zero_acc = [&]() -> int {
        const int blocks = (int)std::min<int64_t>((total + 255) / 256, 8192);
        hipLaunchKernelGGL(psb::k_fill_zero, dim3(blocks), dim3(256), 0, stream, acc, total);
        PSB_HIP_TRY(hipGetLastError());
        return PSB_OK;
    };

    if (fused_segments) {
        int longest = 0;
        for (int i = 0; i < n_seg; ++i) longest = std::max(longest, seg_level[i] - (i ? seg_level[i - 1] : 0));
        const int n_planes = psb::planes_needed(max_shift, longest);
        bool have = ws->ready && ws->ready_seed == seed && ws->ready_layer == layer_id && ws->ready_n_seg == n_seg;
        for (int i = 0; have && i < n_seg; ++i) have = ws->ready_level[i] == seg_level[i];
        ws->ready = false;
        if (!have) {
            rc = sample_segments(q, sp, seg_level, n_seg, seed, layer_id, n_planes, stream);
            if (rc != PSB_OK) return rc;
        }
        if (transpose_blocks > 0) {                 // the layout copy alone
            if (transpose_blocks > 2147483647ll) return PSB_ERR_TOO_LARGE;
            psb::FilterJob none;
            std::memset(&none, 0, sizeof(none));
            hipLaunchKernelGGL(psb::k_shared_prologue, dim3((unsigned)transpose_blocks), dim3(256), 0, stream, none, tj, 0u);
            PSB_HIP_TRY(hipGetLastError());
        }
        p.n_seg = n_seg;
        for (int i = 0; i < 4; ++i) p.seg_level[i] = seg_level[i];
        p.seg_stride = (uint64_t)planes_segment_bytes(sp);
        p.masked = 0;
        int slot = 0;
        const bool timed = profile_begin(stream, &slot);
        psb::launch_conv_shared_mfma(p, n_planes, 0, half_tiles, stream);
        if (timed) profile_end(stream, slot);
        PSB_HIP_TRY(hipGetLastError());
        return PSB_OK;
    }

    if (!budget_to) {
        rc = prepare(0, S);
        if (rc != PSB_OK) return rc;
        if (p.ksplit > 1) {                         // partial sums meet in acc: start from zero, rescale afterwards
            rc = zero_acc();
            if (rc != PSB_OK) return rc;
        }
        rc = contract(S);
        if (rc != PSB_OK) return rc;
        if (p.ksplit > 1 && (y || rq)) return rescale_pass();
        return PSB_OK;
    }

    // per-pixel budgets: the distinct clamped budget values cut the sample axis into segments
    uint32_t present[256];
    if (n_announced > 0) {                          // announced by the caller: nothing to read back
        std::memset(present, 0, sizeof(present));
        for (int i = 0; i < n_announced; ++i) present[std::min<int>(announced[i], q->s_max)] = 1u;
        if (!budget_from) present[0] = 1u;
    } else {
        PSB_HIP_TRY(hipMemsetAsync(ws->present_dev, 0, sizeof(present), stream));
        const int blocks = (int)std::min<int64_t>((npix + 255) / 256, 1024);
        hipLaunchKernelGGL(psb::k_budget_levels, dim3(blocks), dim3(256), 0, stream, budget_to, budget_from, npix,
                           q->s_max, ws->present_dev);
        PSB_HIP_TRY(hipGetLastError());
        PSB_HIP_TRY(hipMemcpyAsync(present, ws->present_dev, sizeof(present), hipMemcpyDeviceToHost, stream));
        PSB_HIP_TRY(hipStreamSynchronize(stream));
    }
    if (!budget_from) {
        rc = zero_acc();
        if (rc != PSB_OK) return rc;
    }
    p.masked = 1;
    int prev = -1;
    for (int v = 0; v < 256; ++v) {
        if (!present[v]) continue;
        if (prev >= 0) {
            p.seg_from = prev; p.seg_to = v;
            rc = prepare(prev, v);
            if (rc != PSB_OK) return rc;
            rc = contract(v - prev);
            if (rc != PSB_OK) return rc;
        }
        prev = v;
    }
    if (y || rq) return rescale_pass();
    return PSB_OK;
}

}  // namespace

extern "C" {

int psb_last_device_error(void) { return tl_last_device_error; }

#ifndef PSB_BUILD_ID
#define PSB_BUILD_ID "unknown"
#endif
const char* psb_build_id(void) { return PSB_BUILD_ID; }

int psb_set_mapping(int mapping)
{
    const int prev = g_mapping;
    if (mapping >= 0 && mapping <= 3) g_mapping = mapping;
    return prev;
}

int psb_shared_window_slots(int32_t kh, int32_t kw, const psb_conv_geom* geom, int32_t half_tiles)
{
    if (!geom) return PSB_ERR_NULL;
    if (kh <= 0 || kw <= 0 || geom->h <= 0 || geom->w <= 0 || geom->stride_h <= 0 || geom->stride_w <= 0 || geom->pad_h < 0 ||
        geom->pad_w < 0 || half_tiles < 1 || half_tiles > 2)
        return PSB_ERR_SHAPE;
    return psb::window_slots(kh, kw, geom->stride_h, geom->stride_w, geom->pad_h, geom->pad_w, geom->h, geom->w, half_tiles);
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
    if (prob_bits < 1 || prob_bits > 23) return PSB_ERR_VALUE;
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
    q->ws = new (std::nothrow) shared_workspace;
    if (!q->ws) { delete q; return PSB_ERR_ALLOC; }
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
    // set-up of the static scratch array of this device (psb_conv2d_requant_static): its address is looked up here,
    // outside any stream capture, so that the entry point itself finds it ready
    {
        const int rc_scratch = static_scratch(q->device, nullptr);
        if (rc_scratch != PSB_OK) return fail(rc_scratch, hipSuccess);
    }
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
        const dim3 grid((unsigned)((K + 63) / 64), (unsigned)(oc_pad / 64));
        if (grid.y > 65535) return fail(PSB_ERR_TOO_LARGE, hipSuccess);
        hipLaunchKernelGGL(psb::k_pack, grid, dim3(256), 0, stream, w_bits, OC, (int)K, oc_pad, (int)prob_bits,
                           field_min, q->packed_dev, q->tile_dev, reinterpret_cast<unsigned long long*>(scratch + 2));
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
    if (q->ws) {
        if (q->ws->w32_dev) (void)hipFree(q->ws->w32_dev);
        if (q->ws->planes_dev) (void)hipFree(q->ws->planes_dev);
        if (q->ws->xt_dev) (void)hipFree(q->ws->xt_dev);
        if (q->ws->present_dev) (void)hipFree(q->ws->present_dev);
        if (q->ws->qmap_dev) (void)hipFree(q->ws->qmap_dev);
        if (q->ws->acc_dev) (void)hipFree(q->ws->acc_dev);
        delete q->ws;
    }
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

int psb_sample_filter(const psb_weights_t* q, int32_t sample_from, int32_t sample_to, uint64_t seed,
                      uint32_t layer_id, int32_t* w_dev, void* hip_stream)
{
    if (!q || !w_dev) return PSB_ERR_NULL;
    if (sample_from < 0 || sample_to <= sample_from || sample_to > q->s_max) return PSB_ERR_VALUE;
    return sample_filter_launch(q, sample_from, sample_to, seed, layer_id, w_dev, nullptr, 1, 1,
                                (hipStream_t)hip_stream);
}

int psb_linear_shared(const psb_weights_t* q, const int8_t* x_dev, int32_t B, int32_t S, uint64_t seed,
                      uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev, const float* bias_dev,
                      void* hip_stream)
{
    if (!q || !x_dev || !acc_dev) return PSB_ERR_NULL;
    if (q->shape.kh != 1 || q->shape.kw != 1 || q->shape.groups != 1) return PSB_ERR_SHAPE;
    if (B <= 0) return PSB_ERR_SHAPE;
    if (S <= 0 || S > q->s_max) return PSB_ERR_VALUE;
    psb_conv_geom g = {B, 1, 1, 1, 1, 0, 0};
    return launch_shared(q, x_dev, &g, S, nullptr, nullptr, seed, layer_id, acc_dev, y_dev, mult_dev, bias_dev,
                         (hipStream_t)hip_stream);
}

int psb_conv2d_shared(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom, int32_t S, uint64_t seed,
                      uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev, const float* bias_dev,
                      void* hip_stream)
{
    if (!q || !x_dev || !geom || !acc_dev) return PSB_ERR_NULL;
    if (S <= 0 || S > q->s_max) return PSB_ERR_VALUE;
    return launch_shared(q, x_dev, geom, S, nullptr, nullptr, seed, layer_id, acc_dev, y_dev, mult_dev, bias_dev,
                         (hipStream_t)hip_stream);
}

int psb_conv2d_progressive_shared(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom,
                                  const uint8_t* budget_to_dev, const uint8_t* budget_from_dev, uint64_t seed,
                                  uint32_t layer_id, int32_t* acc_dev, float* y_dev, const float* mult_dev,
                                  const float* bias_dev, void* hip_stream)
{
    if (!q || !x_dev || !geom || !budget_to_dev || !acc_dev) return PSB_ERR_NULL;
    return launch_shared(q, x_dev, geom, 0, budget_to_dev, budget_from_dev, seed, layer_id, acc_dev, y_dev, mult_dev,
                         bias_dev, (hipStream_t)hip_stream);
}

int psb_conv2d_requant(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom, int32_t S,
                       const uint8_t* budget_to_dev, uint64_t seed, uint32_t layer_id, int32_t* acc_dev, float* y_dev,
                       const float* mult_dev, const float* bias_dev, const psb_requant* rq, int8_t* x_out_dev,
                       int32_t shared, void* hip_stream)
{
    if (!q || !x_dev || !geom || !rq || !x_out_dev) return PSB_ERR_NULL;
    if (!budget_to_dev && (S <= 0 || S > q->s_max)) return PSB_ERR_VALUE;
    if (rq->res_f32_dev && rq->res_i8_dev) return PSB_ERR_VALUE;
    if (rq->lo < -128 || rq->hi > 127 || rq->lo > rq->hi || !(rq->inv_step >= 0.0f)) return PSB_ERR_VALUE;
    psb::Requant r;
    std::memset(&r, 0, sizeof(r));
    r.x_out = x_out_dev; r.res_f32 = rq->res_f32_dev; r.res_i8 = rq->res_i8_dev; r.res_step = rq->res_step;
    r.inv_step = rq->inv_step; r.lo = (float)rq->lo; r.hi = (float)rq->hi; r.relu = rq->relu;
    if (shared)
        return launch_shared(q, x_dev, geom, budget_to_dev ? 0 : S, budget_to_dev, nullptr, seed, layer_id, acc_dev, y_dev,
                             mult_dev, bias_dev, (hipStream_t)hip_stream, &r);
    return launch_layer(q, x_dev, geom, budget_to_dev ? 0 : S, budget_to_dev, nullptr, seed, layer_id, acc_dev, y_dev,
                        mult_dev, bias_dev, (hipStream_t)hip_stream, &r);
}

int psb_conv2d_requant_static(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom, int32_t S,
                              const uint8_t* budget_to_dev, uint64_t seed, uint32_t layer_id, float* y_dev,
                              const float* mult_dev, const float* bias_dev, const psb_requant* rq, int8_t* x_out_dev,
                              void* hip_stream)
{
    if (!q || !x_dev || !geom || !rq || !x_out_dev) return PSB_ERR_NULL;
    if (!budget_to_dev && (S <= 0 || S > q->s_max)) return PSB_ERR_VALUE;
    if (rq->res_f32_dev && rq->res_i8_dev) return PSB_ERR_VALUE;
    if (rq->lo < -128 || rq->hi > 127 || rq->lo > rq->hi || !(rq->inv_step >= 0.0f)) return PSB_ERR_VALUE;
    psb::Requant r;
    std::memset(&r, 0, sizeof(r));
    r.x_out = x_out_dev; r.res_f32 = rq->res_f32_dev; r.res_i8 = rq->res_i8_dev; r.res_step = rq->res_step;
    r.inv_step = rq->inv_step; r.lo = (float)rq->lo; r.hi = (float)rq->hi; r.relu = rq->relu;
    return launch_layer(q, x_dev, geom, budget_to_dev ? 0 : S, budget_to_dev, nullptr, seed, layer_id, nullptr, y_dev,
                        mult_dev, bias_dev, (hipStream_t)hip_stream, &r, /*use_static_scratch=*/true);
}

int psb_conv2d_shared_requant_blocked(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom, int32_t S,
                                      uint64_t seed, uint32_t layer_id, float* y_dev, const float* mult_dev,
                                      const float* bias_dev, const psb_requant* rq, int8_t* x_out_dev, int32_t layout,
                                      void* hip_stream)
{
    if (!q || !x_dev || !geom || (!y_dev && !x_out_dev) || (x_out_dev && !rq)) return PSB_ERR_NULL;
    if (S <= 0 || S > q->s_max) return PSB_ERR_VALUE;
    if (layout & ~(PSB_BLOCKED_IN | PSB_BLOCKED_OUT | PSB_BLOCKED_RES)) return PSB_ERR_VALUE;
    if (!x_out_dev)         // the rescaled values only
        return launch_shared(q, x_dev, geom, S, nullptr, nullptr, seed, layer_id, nullptr, y_dev, mult_dev, bias_dev,
                             (hipStream_t)hip_stream, nullptr, layout & PSB_BLOCKED_IN);
    if (rq->res_f32_dev && rq->res_i8_dev) return PSB_ERR_VALUE;
    if (rq->lo < -128 || rq->hi > 127 || rq->lo > rq->hi || !(rq->inv_step >= 0.0f)) return PSB_ERR_VALUE;
    psb::Requant r;
    std::memset(&r, 0, sizeof(r));
    r.x_out = x_out_dev; r.res_f32 = rq->res_f32_dev; r.res_i8 = rq->res_i8_dev; r.res_step = rq->res_step;
    r.inv_step = rq->inv_step; r.lo = (float)rq->lo; r.hi = (float)rq->hi; r.relu = rq->relu;
    r.out_blocked = (layout & PSB_BLOCKED_OUT) != 0;
    r.res_blocked = (layout & PSB_BLOCKED_RES) != 0 && rq->res_i8_dev;
    return launch_shared(q, x_dev, geom, S, nullptr, nullptr, seed, layer_id, nullptr, y_dev, mult_dev, bias_dev,
                         (hipStream_t)hip_stream, &r, layout);
}

int psb_shared_budget_levels(const uint8_t* levels_host, int32_t n)
{
    if (n < 0 || n > 256) return PSB_ERR_SHAPE;
    if (n > 0 && !levels_host) return PSB_ERR_NULL;
    for (int i = 0; i < n; ++i) tl_levels[i] = levels_host[i];
    tl_levels_n = n;
    return PSB_OK;
}

// Digit planes of n handles sampled ahead of their calls, for the segments [0, l_1), [l_1, l_2), ... of the sample axis.
static int prepare_filters(const psb_weights_t* const* handles, int32_t n, const uint8_t* levels, int32_t n_levels,
                           const uint64_t* seeds, const uint32_t* layer_ids, hipStream_t stream)
{
    int dev = 0;
    PSB_HIP_TRY(hipGetDevice(&dev));
    psb::FilterBatch batch;
    int n_jobs = 0;
    int64_t blocks = 0;
    auto reset = [&]() {
        std::memset(&batch, 0, sizeof(batch));
        for (int k = 0; k <= psb::kMaxBatchJobs; ++k) batch.first_block[k] = 0xFFFFFFFFu;
        n_jobs = 0;
        blocks = 0;
    };
    auto flush = [&]() -> int {
        if (n_jobs == 0) return PSB_OK;
        hipLaunchKernelGGL(psb::k_sample_planes_batch, dim3((unsigned)blocks), dim3(256), 0, stream, batch);
        PSB_HIP_TRY(hipGetLastError());
        reset();
        return PSB_OK;
    };
    reset();
    for (int i = 0; i < n; ++i) {
        const psb_weights* q = handles[i];
        if (q->device != dev) return PSB_ERR_DEVICE;
        const shared_plan sp = plan_shared(q);
        if (!sp.mfma) continue;                 // the direct kernel samples its filter in the call itself
        int level[4] = {0, 0, 0, 0};
        const int n_seg = normalise_levels(levels, n_levels, q->s_max, level);
        if (n_seg <= 0) return PSB_ERR_VALUE;   // no level above 0, or more than four
        if ((int64_t)sp.n_ksteps * 32 * n_seg >= (1ll << 17)) continue;    // the call takes its segments one at a time
        int rc = ensure_planes(q, sp, n_seg, stream);
        if (rc != PSB_OK) return rc;
        int longest = 0;
        for (int k = 0; k < n_seg; ++k) longest = std::max(longest, level[k] - (k ? level[k - 1] : 0));
        const int n_planes = psb::planes_needed(q->info.e_top - q->info.e_min, longest);
        const int64_t need = ((int64_t)sp.n_ocb * sp.n_ksteps + psb::kPlaneGroup - 1) / psb::kPlaneGroup * 4;
        if (need > 2147483647ll) return PSB_ERR_TOO_LARGE;
        for (int k = 0; k < n_seg; ++k) {
            if (n_jobs == psb::kMaxBatchJobs || blocks + need > 2147483647ll) {
                rc = flush();
                if (rc != PSB_OK) return rc;
            }
            psb::FilterJob fj = filter_job(q, k ? level[k - 1] : 0, level[k], seeds[i], layer_ids[i], nullptr,
                                           q->ws->planes_dev + planes_segment_bytes(sp) * k, sp.CB, sp.n_ksteps);
            fj.n_planes = n_planes;
            if (sp.rowpack) { fj.pack_KW = q->shape.kw; fj.pack_C = q->shape.cin; fj.inv_pack_C = psb::inverse_of((uint32_t)q->shape.cin); }
            batch.jobs[n_jobs] = fj;
            batch.first_block[n_jobs] = (unsigned)blocks;
            n_jobs++;
            blocks += need;
        }
        q->ws->ready = true; q->ws->ready_seed = seeds[i]; q->ws->ready_layer = layer_ids[i];
        q->ws->ready_n_seg = n_seg;
        for (int k = 0; k < 4; ++k) q->ws->ready_level[k] = level[k];
    }
    return flush();
}

int psb_shared_prepare_filters(const psb_weights_t* const* handles, int32_t n, int32_t S, const uint64_t* seeds,
                               const uint32_t* layer_ids, void* hip_stream)
{
    if (!handles || !seeds || !layer_ids) return PSB_ERR_NULL;
    if (n <= 0) return PSB_ERR_SHAPE;
    for (int i = 0; i < n; ++i) {
        if (!handles[i]) return PSB_ERR_NULL;
        if (S <= 0 || S > handles[i]->s_max) return PSB_ERR_VALUE;
    }
    const uint8_t level = (uint8_t)S;
    return prepare_filters(handles, n, &level, 1, seeds, layer_ids, (hipStream_t)hip_stream);
}

int psb_shared_prepare_filters_levels(const psb_weights_t* const* handles, int32_t n, const uint8_t* levels_host,
                                      int32_t n_levels, const uint64_t* seeds, const uint32_t* layer_ids, void* hip_stream)
{
    if (!handles || !seeds || !layer_ids || !levels_host) return PSB_ERR_NULL;
    if (n <= 0 || n_levels <= 0 || n_levels > 256) return PSB_ERR_SHAPE;
    for (int i = 0; i < n; ++i)
        if (!handles[i]) return PSB_ERR_NULL;
    return prepare_filters(handles, n, levels_host, n_levels, seeds, layer_ids, (hipStream_t)hip_stream);
}

int psb_conv2d_shared_budget_requant_blocked(const psb_weights_t* q, const int8_t* x_dev, const psb_conv_geom* geom,
                                             const uint8_t* budget_to_dev, const uint8_t* levels_host, int32_t n_levels,
                                             uint64_t seed, uint32_t layer_id, float* y_dev, const float* mult_dev,
                                             const float* bias_dev, const psb_requant* rq, int8_t* x_out_dev,
                                             int32_t layout, void* hip_stream)
{
    if (!q || !x_dev || !geom || !budget_to_dev || !levels_host || (!y_dev && !x_out_dev) || (x_out_dev && !rq))
        return PSB_ERR_NULL;
    if (n_levels <= 0 || n_levels > 256) return PSB_ERR_SHAPE;
    if (layout & ~(PSB_BLOCKED_IN | PSB_BLOCKED_OUT | PSB_BLOCKED_RES)) return PSB_ERR_VALUE;
    {
        int level[4];
        if (normalise_levels(levels_host, n_levels, q->s_max, level) < 0) return PSB_ERR_VALUE;     // more than four
    }
    if (!x_out_dev)         // the rescaled values only
        return launch_shared(q, x_dev, geom, 0, budget_to_dev, nullptr, seed, layer_id, nullptr, y_dev, mult_dev, bias_dev,
                             (hipStream_t)hip_stream, nullptr, layout & PSB_BLOCKED_IN, levels_host, n_levels);
    if (rq->res_f32_dev && rq->res_i8_dev) return PSB_ERR_VALUE;
    if (rq->lo < -128 || rq->hi > 127 || rq->lo > rq->hi || !(rq->inv_step >= 0.0f)) return PSB_ERR_VALUE;
    psb::Requant r;
    std::memset(&r, 0, sizeof(r));
    r.x_out = x_out_dev; r.res_f32 = rq->res_f32_dev; r.res_i8 = rq->res_i8_dev; r.res_step = rq->res_step;
    r.inv_step = rq->inv_step; r.lo = (float)rq->lo; r.hi = (float)rq->hi; r.relu = rq->relu;
    r.out_blocked = (layout & PSB_BLOCKED_OUT) != 0;
    r.res_blocked = (layout & PSB_BLOCKED_RES) != 0 && rq->res_i8_dev;
    return launch_shared(q, x_dev, geom, 0, budget_to_dev, nullptr, seed, layer_id, nullptr, y_dev, mult_dev, bias_dev,
                         (hipStream_t)hip_stream, &r, layout, levels_host, n_levels);
}

// ---- glue between layers ------------------------------------------------------------------------------

int psb_requantize(const float* y_dev, const float* res_f32_dev, const int8_t* res_i8_dev, float res_step, int32_t relu,
                   float inv_step, int32_t lo, int32_t hi, int64_t n, int8_t* x_dev, void* hip_stream)
{
    if (!y_dev || !x_dev) return PSB_ERR_NULL;
    if (n <= 0) return PSB_ERR_SHAPE;
    if (res_f32_dev && res_i8_dev) return PSB_ERR_VALUE;
    if (lo < -128 || hi > 127 || lo > hi || !(inv_step >= 0.0f)) return PSB_ERR_VALUE;
    hipStream_t stream = (hipStream_t)hip_stream;
    const uintptr_t bits = (uintptr_t)y_dev | (uintptr_t)res_f32_dev;
    const bool vec = (bits & 15u) == 0 && (((uintptr_t)res_i8_dev | (uintptr_t)x_dev) & 3u) == 0;
    const int64_t work = vec ? (n + 3) / 4 : n;
    const int blocks = (int)std::min<int64_t>((work + 255) / 256, 16384);
    if (vec)
        hipLaunchKernelGGL(psb::k_requantize<true>, dim3(blocks), dim3(256), 0, stream, y_dev, res_f32_dev, res_i8_dev,
                           res_step, (int)relu, inv_step, (float)lo, (float)hi, n, x_dev);
    else
        hipLaunchKernelGGL(psb::k_requantize<false>, dim3(blocks), dim3(256), 0, stream, y_dev, res_f32_dev, res_i8_dev,
                           res_step, (int)relu, inv_step, (float)lo, (float)hi, n, x_dev);
    PSB_HIP_TRY(hipGetLastError());
    return PSB_OK;
}

int psb_maxpool2d_i8(const int8_t* x_dev, int32_t n, int32_t c, int32_t h, int32_t w, int32_t kh, int32_t kw,
                     int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int8_t* out_dev, void* hip_stream)
{
    if (!x_dev || !out_dev) return PSB_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || kh <= 0 || kw <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 ||
        pad_w < 0)
        return PSB_ERR_SHAPE;
    // every window must contain at least one position of the image
    if (2 * (int64_t)pad_h > kh || 2 * (int64_t)pad_w > kw || (int64_t)h + 2ll * pad_h < kh ||
        (int64_t)w + 2ll * pad_w < kw)
        return PSB_ERR_SHAPE;
    const int64_t OH = ((int64_t)h + 2ll * pad_h - kh) / stride_h + 1, OW = ((int64_t)w + 2ll * pad_w - kw) / stride_w + 1;
    const int64_t images = (int64_t)n * c;
    if (images * h * w >= (1ll << 40) || OH > 2147483647ll || OW > 2147483647ll) return PSB_ERR_TOO_LARGE;
    if (kh == 3 && kw == 3 && stride_h == 2 && stride_w == 2 && pad_h == 1 && pad_w == 1 && w % 4 == 0 && OW % 4 == 0 &&
        (((uintptr_t)x_dev | (uintptr_t)out_dev) & 3u) == 0) {
        const int64_t work = images * OH * (OW / 4);
        hipLaunchKernelGGL(psb::k_maxpool_3x3s2p1_i8, dim3((unsigned)std::min<int64_t>((work + 255) / 256, 65536)), dim3(256),
                           0, (hipStream_t)hip_stream, x_dev, images, h, w, (int)OH, (int)OW, out_dev);
        PSB_HIP_TRY(hipGetLastError());
        return PSB_OK;
    }
    const int64_t total = images * OH * ((OW + 3) / 4);
    const int blocks = (int)std::min<int64_t>((total + 255) / 256, 65536);
    hipLaunchKernelGGL(psb::k_maxpool_i8, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, x_dev, images, h, w, kh, kw,
                       stride_h, stride_w, pad_h, pad_w, (int)OH, (int)OW, (int)(((uintptr_t)out_dev & 3u) == 0), out_dev);
    PSB_HIP_TRY(hipGetLastError());
    return PSB_OK;
}

int psb_maxpool2d_i8_blocked(const int8_t* x_dev, int32_t n, int32_t c, int32_t h, int32_t w, int32_t kh, int32_t kw,
                             int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int8_t* out_dev,
                             void* hip_stream)
{
    if (!x_dev || !out_dev) return PSB_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || kh <= 0 || kw <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 ||
        pad_w < 0)
        return PSB_ERR_SHAPE;
    if (2 * (int64_t)pad_h > kh || 2 * (int64_t)pad_w > kw || (int64_t)h + 2ll * pad_h < kh ||
        (int64_t)w + 2ll * pad_w < kw)
        return PSB_ERR_SHAPE;
    if ((((uintptr_t)x_dev | (uintptr_t)out_dev) & 15u) != 0) return PSB_ERR_VALUE;
    const int64_t OH = ((int64_t)h + 2ll * pad_h - kh) / stride_h + 1, OW = ((int64_t)w + 2ll * pad_w - kw) / stride_w + 1;
    const int64_t cb = ((int64_t)c + 31) / 32;
    if ((int64_t)n * cb * 32 * h * w >= (1ll << 40) || OH > 2147483647ll || OW > 2147483647ll || cb > 2147483647ll)
        return PSB_ERR_TOO_LARGE;
    const int64_t total = (int64_t)n * OH * cb * OW * 2;
    const int blocks = (int)std::min<int64_t>((total + 255) / 256, 65536);
    hipLaunchKernelGGL(psb::k_maxpool_blocked_i8, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, x_dev, n, (int)cb, h, w,
                       kh, kw, stride_h, stride_w, pad_h, pad_w, (int)OH, (int)OW, out_dev);
    PSB_HIP_TRY(hipGetLastError());
    return PSB_OK;
}

int psb_global_avgpool_requantize(const int8_t* x_dev, int32_t n, int32_t c, int32_t h, int32_t w, float scale,
                                  int32_t lo, int32_t hi, int8_t* out_dev, void* hip_stream)
{
    if (!x_dev || !out_dev) return PSB_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return PSB_ERR_SHAPE;
    if ((int64_t)h * w > (1 << 23)) return PSB_ERR_TOO_LARGE;     // the int32 sum and its conversion stay exact
    if (lo < -128 || hi > 127 || lo > hi) return PSB_ERR_VALUE;
    const int64_t images = (int64_t)n * c;
    const int64_t blocks = (images + 3) / 4;
    if (blocks > 2147483647ll) return PSB_ERR_TOO_LARGE;
    const float inv_count = 1.0f / (float)(h * w);                 // correctly rounded division on the host
    hipLaunchKernelGGL(psb::k_avgpool_requantize, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream, x_dev,
                       images, h * w, inv_count, scale, (float)lo, (float)hi, out_dev);
    PSB_HIP_TRY(hipGetLastError());
    return PSB_OK;
}

int psb_budget_resample(const uint8_t* in_dev, int32_t n, int32_t h, int32_t w, int32_t oh, int32_t ow,
                        uint8_t* out_dev, void* hip_stream)
{
    if (!in_dev || !out_dev) return PSB_ERR_NULL;
    if (n <= 0 || h <= 0 || w <= 0 || oh <= 0 || ow <= 0) return PSB_ERR_SHAPE;
    const int64_t total = (int64_t)n * oh * ow;
    const int blocks = (int)std::min<int64_t>((total + 255) / 256, 65536);
    hipLaunchKernelGGL(psb::k_budget_resample, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, in_dev, n, h, w, oh,
                       ow, out_dev);
    PSB_HIP_TRY(hipGetLastError());
    return PSB_OK;
}

int psb_attention_budget(const int8_t* act_dev, float step, int32_t n, int32_t c, int32_t h, int32_t w,
                         uint8_t budget_lo, uint8_t budget_hi, float* entropy_dev, float* mean_dev, uint8_t* budget_dev,
                         void* hip_stream)
{
    if (!act_dev || !entropy_dev || !budget_dev) return PSB_ERR_NULL;
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return PSB_ERR_SHAPE;
    if (!(step > 0.0f) || !(step <= 1e30f)) return PSB_ERR_VALUE;
    const int64_t HW = (int64_t)h * w;
    const int64_t total = (int64_t)n * HW;
    hipStream_t stream = (hipStream_t)hip_stream;
    const int blocks = (int)std::min<int64_t>((total + 255) / 256, 65536);
    hipLaunchKernelGGL(psb::k_channel_entropy, dim3(blocks), dim3(256), 0, stream, act_dev, step, n, c, HW, entropy_dev);
    PSB_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(psb::k_attention_mask, dim3((unsigned)n), dim3(256), 0, stream, entropy_dev, HW, budget_lo,
                       budget_hi, mean_dev, budget_dev);
    PSB_HIP_TRY(hipGetLastError());
    return PSB_OK;
}

}  // extern "C"
