// Suffix prefill attention on the gfx950 matrix cores: bf16 operands, fp32 accumulation.
//
// App. E.4 of the paper: only the uncached suffix is computed and it attends to all stitched
// table content (no mask) and causally to itself.  Because every row of one KV head - all
// suffix tokens times all G query heads of the group - reads the same keys and values, the
// rows are packed into one M dimension (row = token * G + head_in_group): a K/V tile is
// fetched once per KV head and shared by G*S rows, which is what makes the op compute-bound.
//
// Work-group: 4 waves, 128 rows, key tiles of 64 (= 4 pool blocks).  Each wave owns 32 rows and
// computes the TRANSPOSED score tile S^T[key][row] = K . Q^T with v_mfma_f32_32x32x16_bf16, so
// that every lane holds scores of ONE row (column l%32 of the accumulator): row max, row sum and
// the output rescale need no cross-lane traffic except one exchange between lanes l and l^32.
// The exponentials, packed to bf16, are directly the B operand of O^T[d][row] += V^T . P^T; the
// pool stores V transposed inside a block with the token order the operand wants (kv_stitch.hip).
#include "tc_internal.h"

namespace tc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kKRow = 272;            // LDS bytes per K row: 256 + 16 pad (conflict-free b128 reads)
constexpr int kHeadBlk = 4096;        // bytes of one head's K (or V) in one block: 16 * 128 * 2
constexpr float kRescaleThresh = 8.f; // log2 units: rescale O only when the max grew by more

__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(Geom g, BatchDev b, AttnArgs a)
{
    __shared__ __attribute__((aligned(16))) char lds_k[kAttnKeys * kKRow];
    __shared__ __attribute__((aligned(16))) char lds_v[4 * kHeadBlk];

    const AttnItem it = a.items[blockIdx.x];
    if (it.q < 0) return;                              // padding item (uniform for the work-group)
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r32 = lane & 31, hh = lane >> 5;
    const int i = it.q, G = g.G;
    const int P = b.prefix_len[i], S = b.suffix_len[i], cu = b.cu_seqlens[i];
    const int n_blk = (P + S + kBlockTokens - 1) >> 4;
    const int m_rows = S * G;
    const int row_m = it.m0 + w * 32 + r32;
    const bool valid = row_m < m_rows;
    const int rm = valid ? row_m : m_rows - 1;
    const int s_tok = rm / G;
    const int head = it.kvh * G + (rm - s_tok * G);
    const int limit = P + s_tok;                                    // last visible key of this row
    const int wave_limit_min = P + min(it.m0 + w * 32, m_rows - 1) / G;
    const int32_t *bt = b.block_table + (int64_t)i * b.max_blocks;
    const char *layer_base = g.pool + (int64_t)a.layer * g.layer_stride + (int64_t)it.kvh * kHeadBlk + tid * 16;
    const int64_t v_half = g.block_bytes >> 1;

    // Q^T fragments (B operand): lane (row r32, half hh) holds q[row][16*ks + 8*hh .. +8]
    bf16x8 qf[8];
    {
        const char *qp = (const char *)a.q + ((int64_t)(cu + s_tok) * g.Hq + head) * 256 + hh * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = *(const bf16x8 *)(qp + ks * 32);
    }

    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] = 0.f;
    float m_run = -INFINITY, l_lane = 0.f;
    const float c = a.scale_log2;

    // next tile's K/V chunks, prefetched into registers (named scalars: arrays here end up in scratch)
    uint4 k0, k1, k2, k3, v0, v1, v2, v3;
#define TC_LOAD_BLK(t_, j_, kx_, vx_)                                                             \
    {                                                                                             \
        int jb = (t_) * 4 + (j_);                                                                 \
        jb = jb < n_blk ? jb : n_blk - 1; /* past the end: a valid block, masked below */         \
        const char *src = layer_base + (int64_t)bt[jb] * g.block_bytes;                           \
        kx_ = *(const uint4 *)src;                                                                \
        vx_ = *(const uint4 *)(src + v_half);                                                     \
    }
#define TC_LOAD_TILE(t_) TC_LOAD_BLK(t_, 0, k0, v0) TC_LOAD_BLK(t_, 1, k1, v1) TC_LOAD_BLK(t_, 2, k2, v2) TC_LOAD_BLK(t_, 3, k3, v3)
    char *k_st = lds_k + (tid >> 4) * kKRow + (tid & 15) * 16;
    char *v_st = lds_v + tid * 16;
    const char *k_ld = lds_k + r32 * kKRow + hh * 16;
    const char *v_ld = lds_v + r32 * 32 + hh * 16;

    TC_LOAD_TILE(it.tile_begin)
    for (int t = it.tile_begin; t < it.tile_end; ++t) {
        __syncthreads();                               // previous tile fully consumed
        *(uint4 *)(k_st) = k0;                  *(uint4 *)(v_st) = v0;
        *(uint4 *)(k_st + 16 * kKRow) = k1;     *(uint4 *)(v_st + kHeadBlk) = v1;
        *(uint4 *)(k_st + 32 * kKRow) = k2;     *(uint4 *)(v_st + 2 * kHeadBlk) = v2;
        *(uint4 *)(k_st + 48 * kKRow) = k3;     *(uint4 *)(v_st + 3 * kHeadBlk) = v3;
        __syncthreads();
        if (t + 1 < it.tile_end) { TC_LOAD_TILE(t + 1) }   // in flight during the math below

        // S^T[key][row]: two 32-key blocks, contraction over D = 8 steps of 16
        f32x16 sacc[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[mb][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                const bf16x8 ka = *(const bf16x8 *)(k_ld + mb * 32 * kKRow + ks * 32);
                sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[ks], sacc[mb], 0, 0, 0);
            }

        const int key0 = t * kAttnKeys;
        if (key0 + kAttnKeys - 1 > wave_limit_min) {   // causal edge or ragged tail in this tile
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = key0 + 32 * mb + 8 * (e >> 2) + 4 * hh + (e & 3);
                    if (key > limit) sacc[mb][e] = -INFINITY;
                }
        }
        float mx = sacc[0][0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sacc[0][e]);
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[1][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float mxs = mx * c;
        if (__any(mxs > m_run + kRescaleThresh)) {     // also taken while m_run is still -inf
            const float m_new = fmaxf(m_run, mxs);
            const float alpha = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run - m_new);
            l_lane *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
            m_run = m_new;
        }
        const float neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sacc[mb][e], c, neg_m));
                sacc[mb][e] = p;
                l_lane += p;
            }

        // O^T[d][row] += V^T[d][key] P^T[key][row]: four 16-key groups (one pool block each)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 pf;
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[e] = (__bf16)sacc[kk >> 1][8 * (kk & 1) + e];
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x8 va = *(const bf16x8 *)(v_ld + kk * kHeadBlk + db * 32 * 32);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pf, o[db], 0, 0, 0);
            }
        }
    }

#undef TC_LOAD_TILE
#undef TC_LOAD_BLK
    const float l = l_lane + __shfl_xor(l_lane, 32);
    if (!valid) return;
    const int64_t row = (int64_t)(cu + s_tok) * g.Hq + head;
    if (it.n_splits == 1) {
        const float inv = 1.f / l;
        char *op = (char *)a.out + row * 256 + hh * 8;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (__bf16)(o[db][4 * q4 + e] * inv);
                *(bf16x4 *)(op + (32 * db + 8 * q4) * 2) = v;
            }
    } else {
        const int64_t prow = (int64_t)it.split * b.total_S * g.Hq + row;
        float *op = a.part_o + prow * 128 + hh * 4;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                float4 v = make_float4(o[db][4 * q4], o[db][4 * q4 + 1], o[db][4 * q4 + 2], o[db][4 * q4 + 3]);
                *(float4 *)(op + 32 * db + 8 * q4) = v;
            }
        if (hh == 0) { a.part_ml[prow * 2] = m_run; a.part_ml[prow * 2 + 1] = l; }
    }
}

hipError_t launch_attn_bf16(const Geom &g, const BatchDev &b, const AttnArgs &a, hipStream_t s)
{
    if (a.n_items == 0) return hipSuccess;
    if (g.D != 128 || g.esize != 2) return hipErrorInvalidValue;
    attn_bf16_kernel<<<a.n_items, 256, 0, s>>>(g, b, a);
    return hipGetLastError();
}

}  // namespace tc
