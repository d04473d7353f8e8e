// Measurement probe, not part of libtablecache.so: what do the LDS operand reads of the attention
// matrix phases cost on a chip whose clock is set by its power budget?  Matrix streams fed from LDS
// with one 1 KB fragment per v_mfma_f32_32x32x16_bf16 (32 rows per wave, two waves per SIMD whose
// phases alternate at barriers, as in the long-launch kernel) against one fragment per two
// instructions (64 rows per wave, one wave per SIMD), with and without a softmax-sized block of
// vector work.  The summary of a run is profiles/mfma_valu_overlap_probe.txt.
// Build and run:
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Wno-unused-value -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o /tmp/mfma_lds_feed paper_2601_08743_amd/csrc/probes/mfma_lds_feed.hip && /tmp/mfma_lds_feed
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef const __attribute__((address_space(3))) bf16x8 *lds_frag;

__device__ __forceinline__ void valu3(float &x, float &l, float c, float nm)
{
    asm volatile("v_fma_f32 %0, %0, %2, %3\n\tv_exp_f32 %0, %0\n\tv_add_f32 %1, %1, %0" : "+v"(x), "+v"(l) : "v"(c), "v"(nm));
}
// V: 0 = 2 waves/SIMD, 32 rows each, 1 LDS read per MFMA, phases alternate by barrier (like the product kernel, no VALU)
//    1 = same with VALU phase
//    2 = 1 wave/SIMD, 64 rows, 1 LDS read per 2 MFMAs, no VALU
//    3 = 1 wave/SIMD, 64 rows, VALU interleaved between MFMAs (2 scores per MFMA)
//    4 = 2 waves/SIMD, 32 rows each, no LDS reads (operands stay in registers), VALU phase  (what the LDS reads cost)
template <int V>
__global__ __launch_bounds__(512, 1) void probe(const float *in, float *out, int iters)
{
    extern __shared__ __attribute__((aligned(256))) char lds[];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r32 = lane & 31, hh = lane >> 5;
    for (int i = tid; i < 32768 / 4; i += blockDim.x) ((float *)lds)[i] = in[(i * 7 + 3) & 1023];
    __syncthreads();
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    const uint32_t kb = lds0 + r32 * 256 + ((hh ^ (r32 & 15)) << 4);
    bf16x8 q[2][4];
    for (int r = 0; r < 2; ++r) for (int i = 0; i < 4; ++i) for (int e = 0; e < 8; ++e) q[r][i][e] = (__bf16)in[(lane * 53 + r * 97 + i * 8 + e + 300) & 1023];
    f32x16 o[2][4];
    for (int r = 0; r < 2; ++r) for (int i = 0; i < 4; ++i) for (int e = 0; e < 16; ++e) o[r][i][e] = 0.f;
    float s[64], l = 0.f;
    for (int e = 0; e < 64; ++e) s[e] = in[(lane + e * 7) & 1023];
    const float c = 0.001f, nm = -0.5f;
    const int grp = w >> 2;
    if (V == 0 || V == 1 || V == 4) {
        if (grp) __syncthreads();
        for (int it = 0; it < iters; ++it) {
            bf16x8 fr[5];
            if (V != 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j) fr[j] = *(lds_frag)(uintptr_t)((kb ^ ((j & 7) << 5)) + (j >> 3) * 8192);
            } else {
#pragma unroll
                for (int j = 0; j < 5; ++j) fr[j] = q[1][j & 3];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                if (V != 4 && j + 4 < 32) fr[(j + 4) % 5] = *(lds_frag)(uintptr_t)((kb ^ (((j + 4) & 7) << 5)) + ((j + 4) >> 3) * 8192);
                o[0][j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % 5], q[0][(j >> 2) & 3], o[0][j & 3], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
            if (V == 1 || V == 4) {
#pragma unroll
                for (int e = 0; e < 32; ++e) valu3(s[e], l, c, nm);
#pragma unroll
                for (int e = 0; e < 32; e += 2) asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(l) : "v"(s[e]), "v"(s[e + 1]));
#pragma unroll
                for (int e = 0; e < 32; e += 2) asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(s[e]) : "v"(s[e]), "v"(s[e + 1]));
            }
            __syncthreads();
        }
        if (!grp) __syncthreads();
    } else {
        if (w < 4)
        for (int it = 0; it < iters; ++it) {
            bf16x8 fr[5];
#pragma unroll
            for (int j = 0; j < 4; ++j) fr[j] = *(lds_frag)(uintptr_t)((kb ^ ((j & 7) << 5)) + (j >> 3) * 8192);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                if (j + 4 < 32) fr[(j + 4) % 5] = *(lds_frag)(uintptr_t)((kb ^ (((j + 4) & 7) << 5)) + ((j + 4) >> 3) * 8192);
                o[0][j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % 5], q[0][(j >> 2) & 3], o[0][j & 3], 0, 0, 0);
                if (V == 3) { valu3(s[2 * j], l, c, nm); }
                o[1][j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % 5], q[1][(j >> 2) & 3], o[1][j & 3], 0, 0, 0);
                if (V == 3) {
                    valu3(s[2 * j + 1], l, c, nm);
                    asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(l) : "v"(s[2 * j]), "v"(s[2 * j + 1]));
                    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(s[2 * j]) : "v"(s[2 * j]), "v"(s[2 * j + 1]));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    float acc = l;
    for (int r = 0; r < 2; ++r) for (int i = 0; i < 4; ++i) for (int e = 0; e < 16; ++e) acc += o[r][i][e];
    for (int e = 0; e < 64; ++e) acc += s[e];
    out[blockIdx.x * 512 + tid] = acc;
}

template <int V> void run(const char *name, const float *in, float *out, int iters, double mfma_per_iter_per_simd)
{
    hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    (void)hipFuncSetAttribute((const void *)probe<V>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
    float best = 1e9;
    for (int rep = 0; rep < 6; ++rep) {
        (void)hipEventRecord(e0);
        for (int k = 0; k < 20; ++k) hipLaunchKernelGGL(probe<V>, dim3(256), dim3(512), 65536, 0, in, out, iters);
        (void)hipEventRecord(e1); (void)hipEventSynchronize(e1);
        float ms; (void)hipEventElapsedTime(&ms, e0, e1); if (rep >= 2) best = ms < best ? ms : best;
    }
    const double ns_per_iter = best / 20 * 1e6 / iters;
    printf("%-64s %8.1f us/launch, %7.1f ns per iteration, %6.2f ns per matrix instruction and SIMD\n", name, best / 20 * 1e3, ns_per_iter,
           ns_per_iter / mfma_per_iter_per_simd);
    fflush(stdout);
}

int main()
{
    float *in, *out;
    std::vector<float> h(1024);
    srand(1); for (auto &x : h) { float u = 0; for (int k = 0; k < 12; ++k) u += rand() / (float)RAND_MAX; x = u - 6.f; }
    (void)hipMalloc(&in, 4096); (void)hipMalloc(&out, 256 * 512 * 4);
    (void)hipMemcpy(in, h.data(), 4096, hipMemcpyHostToDevice);
    const int iters = 1500;
    for (int pass = 0; pass < 2; ++pass) {
        run<0>("0: 2 waves/SIMD x 32 rows, LDS read per MFMA, phases by barrier", in, out, iters, 64);
        run<1>("1: same + softmax-like vector phase", in, out, iters, 64);
        run<4>("4: as 1 but operands from registers (no LDS reads)", in, out, iters, 64);
        run<2>("2: 1 wave/SIMD x 64 rows, LDS read per 2 MFMAs", in, out, iters, 64);
        run<3>("3: same + vector work interleaved", in, out, iters, 64);
    }
    return 0;
}
