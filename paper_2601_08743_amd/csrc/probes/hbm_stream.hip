// Measurement probe, not part of libtablecache.so: what can plain streaming kernels move through
// this chip's HBM?  The gather (tc_stitch_kv) and the decode attention kernels are priced against
// the data-sheet 8 TB/s; this gives the figure a kernel that does nothing else reaches, for a
// read-only sweep, a write-only sweep, a copy of contiguous memory, and a copy in pieces of 4 KB
// and 64 KB whose sources are shuffled (the gather's pattern: whole blocks from scattered table
// slots; the decode kernels read 4 KB per head and block).  Buffers of 4 GiB (16 times the 256 MB
// last-level cache).  The summary of a run is profiles/hbm_stream_probe.txt.
// Build and run:
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o /tmp/hbm_stream paper_2601_08743_amd/csrc/probes/hbm_stream.hip && /tmp/hbm_stream
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <numeric>
#include <random>
#include <vector>

#define CHECK(x)                                                                                   \
    do {                                                                                           \
        hipError_t e_ = (x);                                                                       \
        if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); std::exit(1); } \
    } while (0)

// every thread moves 16 bytes per step; a work-group of 256 threads covers 4 KB per step and walks
// `per_wg` consecutive pieces of `piece` bytes, the i-th of them taken from piece perm[i] of the source
__global__ __launch_bounds__(256) void copy_pieces(const uint4 *src, uint4 *dst, const int32_t *perm, int piece16, int per_wg)
{
    for (int k = 0; k < per_wg; ++k) {
        const int64_t p = (int64_t)blockIdx.x * per_wg + k;
        const uint4 *s = src + (int64_t)(perm ? perm[p] : p) * piece16;
        uint4 *d = dst + p * piece16;
        for (int i = threadIdx.x; i < piece16; i += 256) d[i] = s[i];
    }
}
__global__ __launch_bounds__(256) void read_only(const uint4 *src, uint4 *sink, int64_t n16)
{
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) {
        const uint4 v = src[i];
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[threadIdx.x] = acc;     // keeps the loads alive
}
__global__ __launch_bounds__(256) void write_only(uint4 *dst, int64_t n16)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256)
        dst[i] = make_uint4((uint32_t)i, 1, 2, 3);
}

template <typename F>
static double time_ms(F &&launch, int reps)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    launch();
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    for (int r = 0; r < reps; ++r) launch();
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    CHECK(hipGetLastError());
    return ms / reps;
}

int main()
{
    const int64_t bytes = 4ll << 30, n16 = bytes / 16;
    uint4 *a, *b;
    CHECK(hipMalloc(&a, bytes));
    CHECK(hipMalloc(&b, bytes));
    CHECK(hipMemset(a, 0x5a, bytes));
    CHECK(hipMemset(b, 0, bytes));
    const int reps = 10;
    std::printf("%-44s %10s %10s\n", "kernel (4 GiB per buffer)", "ms", "GB/s");
    for (int grid : {256 * 8, 256 * 32}) {
        double ms = time_ms([&] { hipLaunchKernelGGL(read_only, dim3(grid), dim3(256), 0, 0, a, b, n16); }, reps);
        std::printf("read only, %5d work-groups %*s %10.3f %10.0f\n", grid, 17, "", ms, bytes / ms / 1e6);
        ms = time_ms([&] { hipLaunchKernelGGL(write_only, dim3(grid), dim3(256), 0, 0, b, n16); }, reps);
        std::printf("write only, %5d work-groups %*s %10.3f %10.0f\n", grid, 16, "", ms, bytes / ms / 1e6);
    }
    for (int piece : {4096, 65536}) {
        const int64_t n_pieces = bytes / piece;
        std::vector<int32_t> perm(n_pieces);
        std::iota(perm.begin(), perm.end(), 0);
        std::mt19937 rng(7);
        // shuffle runs of 32 pieces (a table's blocks are contiguous in its slot; tables are scattered)
        const int run = 32;
        std::vector<int32_t> runs(n_pieces / run);
        std::iota(runs.begin(), runs.end(), 0);
        std::shuffle(runs.begin(), runs.end(), rng);
        for (int64_t r = 0; r < (int64_t)runs.size(); ++r)
            for (int k = 0; k < run; ++k) perm[r * run + k] = runs[r] * run + k;
        int32_t *d_perm;
        CHECK(hipMalloc(&d_perm, n_pieces * 4));
        CHECK(hipMemcpy(d_perm, perm.data(), n_pieces * 4, hipMemcpyHostToDevice));
        const int per_wg = piece == 4096 ? 16 : 1;
        const int grid = (int)(n_pieces / per_wg);
        double ms = time_ms([&] { hipLaunchKernelGGL(copy_pieces, dim3(grid), dim3(256), 0, 0, a, b, (const int32_t *)nullptr, piece / 16, per_wg); }, reps);
        std::printf("copy, pieces of %6d B in order %*s %10.3f %10.0f   (read + written)\n", piece, 13, "", ms, 2.0 * bytes / ms / 1e6);
        ms = time_ms([&] { hipLaunchKernelGGL(copy_pieces, dim3(grid), dim3(256), 0, 0, a, b, (const int32_t *)d_perm, piece / 16, per_wg); }, reps);
        std::printf("copy, pieces of %6d B, sources shuffled %*s %10.3f %10.0f   (read + written)\n", piece, 4, "", ms, 2.0 * bytes / ms / 1e6);
        CHECK(hipFree(d_perm));
    }
    double ms = time_ms([&] { CHECK(hipMemcpyAsync(b, a, bytes, hipMemcpyDeviceToDevice, 0)); }, reps);
    std::printf("hipMemcpyAsync device to device %*s %10.3f %10.0f   (read + written)\n", 12, "", ms, 2.0 * bytes / ms / 1e6);
    CHECK(hipFree(a));
    CHECK(hipFree(b));
    return 0;
}
