// Suffix prefill attention, fp32 storage and fp32 arithmetic (no reduced-precision operands).
// App. E.4 of the paper: the suffix rows attend to all stitched schema keys, and causally to
// the suffix itself.  Online softmax over key tiles of 64; one wave per (suffix token, head) row,
// four rows per work-group sharing the K tile through LDS.  This variant exists for the fp32
// configuration, which is small and latency-bound; the matrix-core path is the bf16 kernel.
#include "tc_internal.h"

namespace tc {

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(Geom g, BatchDev b, AttnArgs a)
{
    constexpr int DP = D + 1;                    // padded K row: lanes read distinct banks
    constexpr int DPL = D / 64;                  // output columns per lane
    __shared__ float ks[kF32Keys * DP];
    __shared__ float pw[kF32Rows][kF32Keys];
    const AttnItem it = a.items[blockIdx.x];
    if (it.q < 0) return;                              // padding item (uniform for the work-group)
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int i = it.q;
    const int P = b.prefix_len[i], S = b.suffix_len[i], cu = b.cu_seqlens[i];
    const int n_blk = (P + S + kBlockTokens - 1) >> 4;
    const int m = it.m0 + w;
    const bool valid = m < S * g.G;
    const int s_tok = valid ? m / g.G : 0;
    const int head = it.kvh * g.G + (valid ? m % g.G : 0);
    const int limit = P + s_tok;                 // last visible key
    const int32_t *bt = b.block_table + (int64_t)i * b.max_blocks;
    const char *layer_base = g.pool + (int64_t)a.layer * g.layer_stride;
    const int64_t head_off = (int64_t)it.kvh * kBlockTokens * g.head_bytes;

    float qreg[D];
    {
        const float *qp = (const float *)a.q + ((int64_t)(cu + s_tok) * g.Hq + head) * D;
#pragma unroll
        for (int d = 0; d < D; ++d) qreg[d] = qp[d];
    }
    float m_run = -INFINITY, l_lane = 0.f;
    float acc[DPL];
#pragma unroll
    for (int c = 0; c < DPL; ++c) acc[c] = 0.f;

    for (int t = it.tile_begin; t < it.tile_end; ++t) {
        const int key0 = t * kF32Keys;
        __syncthreads();                         // previous tile's readers are done
        // stage K: 4 blocks x 16 tokens x D floats, coalesced rows
        for (int c = tid; c < kF32Keys * (D / 4); c += 256) {
            const int kk = c / (D / 4), d4 = c % (D / 4);
            int jb = (key0 + kk) >> 4;
            jb = jb < n_blk ? jb : n_blk - 1;    // past the end: any valid block, masked below
            const float4 v = *(const float4 *)(layer_base + (int64_t)bt[jb] * g.block_bytes + head_off +
                                               ((int64_t)((key0 + kk) & 15) * D + d4 * 4) * 4);
            float *dst = ks + kk * DP + d4 * 4;
            dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
        }
        __syncthreads();
        // scores: lane <-> key
        const int key = key0 + lane;
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) s = fmaf(qreg[d], ks[lane * DP + d], s);
        s = (key <= limit) ? s * a.scale_log2 : -INFINITY;
        const float m_new = fmaxf(m_run, wave_max(s));
        const float m_eff = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = (m_run == -INFINITY) ? 0.f : exp2f(m_run - m_eff);
        const float p = exp2f(s - m_eff);
        l_lane = l_lane * alpha + p;
        m_run = m_new;
        pw[w][lane] = p;
        __syncthreads();
        // values: lane <-> output column(s); V rows straight from the pool (row-contiguous)
#pragma unroll
        for (int c = 0; c < DPL; ++c) acc[c] *= alpha;
        const int n_here = min(kF32Keys, max(0, min(limit, P + S - 1) - key0 + 1));
        for (int kk = 0; kk < n_here; ++kk) {
            const int jb = (key0 + kk) >> 4;
            const float *vrow = (const float *)(layer_base + (int64_t)bt[jb] * g.block_bytes +
                                                (g.block_bytes >> 1) + head_off) +
                                ((key0 + kk) & 15) * D;
            const float pj = pw[w][kk];
#pragma unroll
            for (int c = 0; c < DPL; ++c) acc[c] = fmaf(pj, vrow[lane + 64 * c], acc[c]);
        }
    }
    const float l = wave_sum(l_lane);
    if (!valid) return;
    const int64_t row = (int64_t)(cu + s_tok) * g.Hq + head;
    if (it.n_splits == 1) {
        float *o = (float *)a.out + row * D;
        const float inv = 1.f / l;
#pragma unroll
        for (int c = 0; c < DPL; ++c) o[lane + 64 * c] = acc[c] * inv;
    } else {
        const int64_t prow = (int64_t)it.split * b.total_S * g.Hq + row;
        float *o = a.part_o + prow * D;
#pragma unroll
        for (int c = 0; c < DPL; ++c) o[lane + 64 * c] = acc[c];
        if (lane == 0) { a.part_ml[prow * 2] = m_run; a.part_ml[prow * 2 + 1] = l; }
    }
}

hipError_t launch_attn_f32(const Geom &g, const BatchDev &b, const AttnArgs &a, const Launch &L)
{
    if (a.n_items == 0) return hipSuccess;
    if (g.D == 64)
        TC_LAUNCH(attn_f32_kernel<64>, a.n_items, 0, L, g, b, a);
    else if (g.D == 128)
        TC_LAUNCH(attn_f32_kernel<128>, a.n_items, 0, L, g, b, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ merge
// Combine split-KV partials of one output row: with reference maxima m_s (log2 units), sums l_s
// and unnormalised partial outputs O_s:  out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// One wave per (suffix token, head) row.
template <typename OutT>
__global__ __launch_bounds__(256) void merge_kernel(Geom g, BatchDev b, AttnArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t n_rows = (int64_t)b.total_S * g.Hq;
    if (row >= n_rows) return;
    const int n = (int)(row / g.Hq);
    const int ns = b.splits_of_q[b.tok_q[n]];
    if (ns <= 1) return;                         // written directly by the attention kernel
    float M = -INFINITY;
    for (int s = 0; s < ns; ++s) M = fmaxf(M, a.part_ml[((int64_t)s * n_rows + row) * 2]);
    float den = 0.f;
    float acc[2] = {0.f, 0.f};
    const int D = g.D;
    for (int s = 0; s < ns; ++s) {
        const int64_t prow = (int64_t)s * n_rows + row;
        const float ms = a.part_ml[prow * 2];
        const float wgt = (ms == -INFINITY) ? 0.f : exp2f(ms - M);
        den += wgt * a.part_ml[prow * 2 + 1];
        const float *o = a.part_o + prow * D;
        for (int c = 0; c * 64 < D; ++c) acc[c] = fmaf(wgt, o[lane + 64 * c], acc[c]);
    }
    const float inv = 1.f / den;
    OutT *o = (OutT *)a.out + row * D;
    for (int c = 0; c * 64 < D; ++c) o[lane + 64 * c] = (OutT)(acc[c] * inv);
}

hipError_t launch_merge(const Geom &g, const BatchDev &b, const AttnArgs &a, const Launch &L)
{
    const int64_t n_rows = (int64_t)b.total_S * g.Hq;
    if (n_rows == 0) return hipSuccess;
    const int grid = (int)((n_rows + 3) / 4);
    if (g.esize == 2)
        TC_LAUNCH(merge_kernel<__bf16>, grid, 0, L, g, b, a);
    else
        TC_LAUNCH(merge_kernel<float>, grid, 0, L, g, b, a);
    return hipGetLastError();
}

}  // namespace tc
