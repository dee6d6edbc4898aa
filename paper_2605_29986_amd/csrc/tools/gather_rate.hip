// Calibration tool for the walk kernels' roofline: the rate at which a kernel that does nothing
// else performs dependent 2-byte table reads tab[b * S + cur] from an L2-resident transposed
// automaton table [256][S], the access pattern of one step of the byte walk (paper Section
// 3.2.1 / Algorithm 1, regular case).  Two patterns: the byte (table column) is the same for a
// whole wave, as when a wave walks the image states of one token; or every lane has its own.
// Prints one line per (S, pattern, reads in flight per thread).
//
//   gather_rate [S ...]        default: 1024 4096

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#define CHECK(x)                                                                    \
    do {                                                                            \
        hipError_t e_ = (x);                                                        \
        if (e_ != hipSuccess) {                                                     \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                               \
        }                                                                           \
    } while (0)

template <int U>
__global__ __launch_bounds__(256) void gather_kernel(const uint16_t *__restrict__ tab, uint32_t S,
                                                     const uint8_t *__restrict__ bytes, int steps,
                                                     uint32_t *out, int wave_uniform_column) {
    uint32_t cur[U];
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
#pragma unroll
    for (int u = 0; u < U; ++u) cur[u] = (gid * 2654435761u + u * 40503u) % S;
    for (int p = 0; p < steps; ++p) {
        const uint32_t who = wave_uniform_column ? (gid >> 6) : gid;
        const uint32_t b = bytes[(who + p * 131u) & 0xFFFFu];
#pragma unroll
        for (int u = 0; u < U; ++u) cur[u] = tab[b * S + cur[u]];
    }
    uint32_t acc = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) acc += cur[u];
    out[gid] = acc;
}

template <int U>
static int run(const uint16_t *tab, uint32_t S, const uint8_t *bytes, uint32_t *out, int uniform) {
    const int blocks = 256 * 8, threads = 256, steps = 64, repeats = 5;
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    hipLaunchKernelGGL(gather_kernel<U>, dim3(blocks), dim3(threads), 0, 0, tab, S, bytes, steps, out, uniform);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    for (int r = 0; r < repeats; ++r)
        hipLaunchKernelGGL(gather_kernel<U>, dim3(blocks), dim3(threads), 0, 0, tab, S, bytes, steps, out, uniform);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double reads = (double)repeats * blocks * threads * steps * U;
    std::printf("{\"S\": %u, \"column\": \"%s\", \"in_flight\": %d, \"reads_per_s\": %.4e}\n", S,
                uniform ? "wave-uniform" : "per-lane", U, reads / (ms * 1e-3));
    std::fflush(stdout);
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return 0;
}

int main(int argc, char **argv) {
    std::vector<uint32_t> sizes;
    for (int i = 1; i < argc; ++i) sizes.push_back((uint32_t)std::atoi(argv[i]));
    if (sizes.empty()) sizes = {1024u, 4096u};
    for (uint32_t S : sizes) {
        if (S == 0 || S > 65536) {
            std::printf("S must be in 1..65536\n");
            return 2;
        }
        std::vector<uint16_t> h((size_t)256 * S);
        std::mt19937 rng(1);
        for (auto &v : h) v = (uint16_t)(rng() % S);
        std::vector<uint8_t> hb(65536);
        for (auto &v : hb) v = (uint8_t)(rng() & 255);
        uint16_t *tab = nullptr;
        uint8_t *bytes = nullptr;
        uint32_t *out = nullptr;
        CHECK(hipMalloc(&tab, h.size() * 2));
        CHECK(hipMalloc(&bytes, hb.size()));
        CHECK(hipMalloc(&out, (size_t)256 * 8 * 256 * 4));
        CHECK(hipMemcpy(tab, h.data(), h.size() * 2, hipMemcpyHostToDevice));
        CHECK(hipMemcpy(bytes, hb.data(), hb.size(), hipMemcpyHostToDevice));
        for (int uniform = 1; uniform >= 0; --uniform) {
            if (run<1>(tab, S, bytes, out, uniform)) return 1;
            if (run<2>(tab, S, bytes, out, uniform)) return 1;
            if (run<4>(tab, S, bytes, out, uniform)) return 1;
            if (run<8>(tab, S, bytes, out, uniform)) return 1;
        }
        CHECK(hipFree(tab));
        CHECK(hipFree(bytes));
        CHECK(hipFree(out));
    }
    return 0;
}
