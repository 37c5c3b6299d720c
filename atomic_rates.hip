// Rate of returnless int32 atomic adds by the layout of a wave's 64 addresses (gfx950).
//
// The channel-lane PSB kernel adds the partial sums of its tap chunks in memory, lane = output channel.  In
// [N][OC][OH][OW] order the 64 adds of a wave go to 64 lines one output plane apart; in [N*OH*OW][OC] order they
// are 64 consecutive words.  This program times both on the shape of a ResNet-18 stage-1 layer (batch 32, 56 x 56,
// 64 channels, 9 chunks: every word is hit 9 times, by different workgroups) and checks the sums.
// Under `rocprofv3 --pmc WRITE_SIZE -- ./atomic_rates` the counter gives the bytes the memory side writes per add.
//
// Build: hipcc --offload-arch=gfx950 -O3 atomic_rates.hip -o atomic_rates ; run: ./atomic_rates
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <vector>

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));              \
            return 2;                                                                 \
        }                                                                             \
    } while (0)

// wave w of workgroup b adds lane + 1 to the 64 channels of pixel 4 b + w, 4 b + w + 4 gridDim.x, ...;
// blockIdx.y = chunk (the same words again)
template <bool CHANNELS_LAST>
__global__ void __launch_bounds__(256) k_adds(int32_t* acc, int npix, int plane)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int pix = blockIdx.x * 4 + wave; pix < npix; pix += gridDim.x * 4) {
        const int n = pix / plane, r = pix - n * plane;
        const size_t idx = CHANNELS_LAST ? (size_t)pix * 64 + lane : ((size_t)n * 64 + lane) * plane + r;
        atomicAdd(&acc[idx], lane + 1);
    }
}

int main()
{
    const int plane = 56 * 56, npix = 32 * plane, chunks = 9;
    const size_t words = (size_t)npix * 64;
    int32_t* acc = nullptr;
    CHECK(hipMalloc(&acc, words * sizeof(int32_t)));
    std::vector<int32_t> host(words);
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int rep = 0; rep < 2; ++rep) {
        for (int last = 0; last < 2; ++last) {
            CHECK(hipMemset(acc, 0, words * sizeof(int32_t)));
            CHECK(hipDeviceSynchronize());
            CHECK(hipEventRecord(e0, 0));
            if (last) hipLaunchKernelGGL(k_adds<true>, dim3(1024, chunks), dim3(256), 0, 0, acc, npix, plane);
            else hipLaunchKernelGGL(k_adds<false>, dim3(1024, chunks), dim3(256), 0, 0, acc, npix, plane);
            CHECK(hipGetLastError());
            CHECK(hipEventRecord(e1, 0));
            CHECK(hipEventSynchronize(e1));
            float ms = 0;
            CHECK(hipEventElapsedTime(&ms, e0, e1));
            CHECK(hipMemcpy(host.data(), acc, words * sizeof(int32_t), hipMemcpyDeviceToHost));
            long long total = 0;
            for (int32_t v : host) total += v;
            const long long expect = (long long)npix * chunks * (64 * 65 / 2);
            const double adds = (double)words * chunks;
            std::printf("%-44s %8.3f ms for %.1f M adds = %6.1f G adds/s, sums %s\n",
                        last ? "[N*OH*OW][OC]: 64 consecutive words per wave" : "[N][OC][OH][OW]: 64 lines, one plane apart",
                        ms, adds / 1e6, adds / ms / 1e6, total == expect ? "ok" : "WRONG");
            if (total != expect) return 1;
        }
    }
    CHECK(hipFree(acc));
    return 0;
}
