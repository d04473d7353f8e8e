// Measurement probe, not part of libtablecache.so: do matrix (MFMA) and vector (VALU) instructions of
// the prefill-attention inner loop overlap on a gfx950 SIMD, and what does the chip's clock do
// meanwhile?  Per iteration 32 v_mfma_f32_32x32x16_bf16 on N(0,1)-like operands and a softmax-sized
// block of vector work (32 x (fma, exp2, add) + 32 max), one work-group per CU on all 256 CUs:
//   0 matrix only, 1 vector only, 2 one after the other in one wave, 3 interleaved in one wave,
//   4 two waves per SIMD: one matrix, one vector, 5 two waves per SIMD, each serial, half a period apart.
// Prints cycles per iteration (s_memtime), wall time per iteration (s_memrealtime) and their ratio,
// the shader clock.  The summary of a run is profiles/mfma_valu_overlap_probe.txt.
// Build and run:
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Wno-unused-value -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o /tmp/mfma_valu_overlap paper_2601_08743_amd/csrc/probes/mfma_valu_overlap.hip && /tmp/mfma_valu_overlap
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void mfma(f32x16 &acc, const bf16x8 &a, const bf16x8 &b)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void valu5(float &x, float &l, float c, float nm, unsigned &pk, float y)
{
    asm volatile("v_fma_f32 %0, %0, %2, %3\n\tv_exp_f32 %0, %0\n\tv_add_f32 %1, %1, %0" : "+v"(x), "+v"(l) : "v"(c), "v"(nm));
}
template <int V>
__global__ __launch_bounds__(512, 1) void probe(const float *in, float *out, unsigned long long *stamps, int iters)
{
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int grp = w >> 2;
    bf16x8 a[4], b[4];
    for (int i = 0; i < 4; ++i)
        for (int e = 0; e < 8; ++e) { a[i][e] = (__bf16)in[(lane * 37 + i * 8 + e) & 1023]; b[i][e] = (__bf16)in[(lane * 53 + i * 8 + e + 300) & 1023]; }
    f32x16 o[4];
    for (int i = 0; i < 4; ++i) for (int e = 0; e < 16; ++e) o[i][e] = 0.f;
    float s[32], l = 0.f;
    for (int e = 0; e < 32; ++e) s[e] = in[(lane + e * 7) & 1023];
    const float c = 0.001f, nm = -0.5f;
    unsigned long long t0, t1, r0, r1;
    asm volatile("s_memtime %0\n\ts_memrealtime %1\n\ts_waitcnt lgkmcnt(0)" : "=s"(t0), "=s"(r0));
    const bool do_m = V == 0 || V == 2 || V == 3 || (V == 4 && grp == 0) || V == 5;
    const bool do_v = V == 1 || V == 2 || V == 3 || (V == 4 && grp == 1) || V == 5;
    if (V == 5 && grp == 1) {            // half a period behind: start with the vector block
#pragma unroll
        for (int e = 0; e < 32; ++e) { unsigned pk; valu5(s[e], l, c, nm, pk, 0.f); }
#pragma unroll
        for (int e = 0; e < 32; ++e) asm volatile("v_max_f32 %0, %0, %1" : "+v"(l) : "v"(s[e]));
    }
    for (int it = 0; it < iters; ++it) {
        if (V == 3) {
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                mfma(o[j & 3], a[j & 3], b[(j >> 2) & 3]);
                unsigned pk; valu5(s[j], l, c, nm, pk, 0.f);
                asm volatile("v_max_f32 %0, %0, %1" : "+v"(l) : "v"(s[j]));
            }
        } else {
            if (do_m) {
#pragma unroll
                for (int j = 0; j < 32; ++j) mfma(o[j & 3], a[j & 3], b[(j >> 2) & 3]);
            }
            if (do_v) {
#pragma unroll
                for (int e = 0; e < 32; ++e) { unsigned pk; valu5(s[e], l, c, nm, pk, 0.f); }
#pragma unroll
                for (int e = 0; e < 32; ++e) asm volatile("v_max_f32 %0, %0, %1" : "+v"(l) : "v"(s[e]));
            }
        }
    }
    asm volatile("s_nop 15\n\ts_memtime %0\n\ts_memrealtime %1\n\ts_waitcnt lgkmcnt(0)" : "=s"(t1), "=s"(r1));
    float acc = l;
    for (int i = 0; i < 4; ++i) for (int e = 0; e < 16; ++e) acc += o[i][e];
    for (int e = 0; e < 32; ++e) acc += s[e];
    out[blockIdx.x * 512 + tid] = acc;
    if (lane == 0) { stamps[(blockIdx.x * 8 + w) * 2] = t1 - t0; stamps[(blockIdx.x * 8 + w) * 2 + 1] = r1 - r0; }
}

template <int V> void run(const char *name, int threads, const float *in, float *out, unsigned long long *st, int iters)
{
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    float best = 1e9;
    for (int rep = 0; rep < 6; ++rep) {
        hipEventRecord(e0);
        for (int k = 0; k < 20; ++k) hipLaunchKernelGGL(probe<V>, dim3(256), dim3(threads), 0, 0, in, out, st, iters);
        hipEventRecord(e1); hipEventSynchronize(e1);
        float ms; hipEventElapsedTime(&ms, e0, e1); if (rep >= 2) best = ms < best ? ms : best;
    }
    std::vector<unsigned long long> h(256 * 8 * 2);
    hipMemcpy(h.data(), st, h.size() * 8, hipMemcpyDeviceToHost);
    double cyc = 0, real = 0; int n = 0;
    for (int b = 0; b < 256; ++b) for (int w = 0; w < threads / 64; ++w) { cyc += h[(b * 8 + w) * 2]; real += h[(b * 8 + w) * 2 + 1]; ++n; }
    cyc /= n; real /= n;
    printf("%-44s %3d thr: %8.1f us/launch, %7.1f cycles/iter, %7.1f ns/iter, clock %.3f GHz\n", name, threads, best / 20 * 1e3,
           cyc / iters, real * 10.0 / iters, cyc / (real * 10.0));
    fflush(stdout);
}

int main()
{
    float *in, *out; unsigned long long *st;
    std::vector<float> h(1024);
    srand(1); for (auto &x : h) { float u = 0; for (int k = 0; k < 12; ++k) u += rand() / (float)RAND_MAX; x = u - 6.f; }
    hipMalloc(&in, 4096); hipMalloc(&out, 256 * 512 * 4); hipMalloc(&st, 256 * 8 * 2 * 8);
    hipMemcpy(in, h.data(), 4096, hipMemcpyHostToDevice);
    const int iters = 2000;
    for (int pass = 0; pass < 2; ++pass) {
        run<0>("0 MFMA only (32 per iter)", 256, in, out, st, iters);
        run<1>("1 VALU only (128 per iter, 32 exp)", 256, in, out, st, iters);
        run<2>("2 serial in one wave", 256, in, out, st, iters);
        run<3>("3 interleaved in one wave", 256, in, out, st, iters);
        run<0>("0 MFMA only, two waves per SIMD", 512, in, out, st, iters);
        run<1>("1 VALU only, two waves per SIMD", 512, in, out, st, iters);
        run<4>("4 two waves: one MFMA, one VALU", 512, in, out, st, iters);
        run<5>("5 two waves, serial, out of phase", 512, in, out, st, iters);
        run<2>("2 two waves, serial, in phase", 512, in, out, st, iters);
        run<3>("3 two waves, interleaved", 512, in, out, st, iters);
    }
    return 0;
}
