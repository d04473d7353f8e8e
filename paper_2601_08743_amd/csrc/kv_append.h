// Suffix append, shared by the stand-alone append kernel (fp32 path) and the bf16 attention
// kernel (which runs it in extra work-groups of its own launch).
#pragma once
#include "tc_internal.h"

namespace tc {

__device__ __forceinline__ int vperm(int t) { return (t & 3) | ((t & 4) << 1) | ((t & 8) >> 1); }

// The suffix tokens' own K/V go to logical positions [P_i, P_i + S_i) of the sequence (pool
// block layout), so the pool holds the whole prompt afterwards.  Work unit n < total_S handles
// suffix token n; unit total_S + i zero-fills the unused tail of query i's last block.
template <bool kTransposeV>
__device__ __forceinline__ void append_unit(const Geom &g, const BatchDev &b, int layer, const char *k_new,
                                            const char *v_new, int n, int tid)
{
    char *layer_base = g.pool + (int64_t)layer * g.layer_stride;
    const int cpr = g.row_bytes >> 4, cph = g.head_bytes >> 4;
    if (n < b.total_S) {
        const int i = b.tok_q[n];
        const int p = b.prefix_len[i] + (n - b.cu_seqlens[i]);
        const int phys = entry_bid(b.block_table[(int64_t)i * b.max_blocks + (p >> 4)]);
        const int t = p & 15;
        char *kd = layer_base + (int64_t)phys * g.block_bytes;
        char *vd = kd + (g.block_bytes >> 1);
        for (int w = tid; w < cpr; w += 256) {
            const int h = w / cph, dc = w - h * cph;
            const uint4 kv = *(const uint4 *)(k_new + (int64_t)n * g.row_bytes + (w << 4));
            *(uint4 *)(kd + (int64_t)(h * kBlockTokens + t) * g.head_bytes + (dc << 4)) = kv;
            const uint4 vv = *(const uint4 *)(v_new + (int64_t)n * g.row_bytes + (w << 4));
            if (!kTransposeV) {
                *(uint4 *)(vd + (int64_t)(h * kBlockTokens + t) * g.head_bytes + (dc << 4)) = vv;
            } else {
                const unsigned u[4] = {vv.x, vv.y, vv.z, vv.w};
                unsigned short *v16 = (unsigned short *)vd;
                const int d0 = dc << 3;            // 8 bf16 per chunk
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const unsigned short e = (unsigned short)(u[k >> 1] >> ((k & 1) * 16));
                    v16[((int64_t)(h * g.D + d0 + k) << 4) + vperm(t)] = e;
                }
            }
        }
    } else {
        const int i = n - b.total_S;
        const int end = b.prefix_len[i] + b.suffix_len[i];
        const int t0 = end & 15;
        if (t0 == 0) return;
        const int phys = entry_bid(b.block_table[(int64_t)i * b.max_blocks + (end >> 4)]);
        char *kd = layer_base + (int64_t)phys * g.block_bytes;
        char *vd = kd + (g.block_bytes >> 1);
        const uint4 zero = make_uint4(0, 0, 0, 0);
        const int n_tail = kBlockTokens - t0;
        for (int c = tid; c < n_tail * cpr; c += 256) {
            const int t = t0 + c / cpr, w = c % cpr;
            const int h = w / cph, dc = w - h * cph;
            *(uint4 *)(kd + (int64_t)(h * kBlockTokens + t) * g.head_bytes + (dc << 4)) = zero;
            if (!kTransposeV) {
                *(uint4 *)(vd + (int64_t)(h * kBlockTokens + t) * g.head_bytes + (dc << 4)) = zero;
            } else {
                unsigned short *v16 = (unsigned short *)vd;
                const int d0 = dc << 3;
#pragma unroll
                for (int k = 0; k < 8; ++k) v16[((int64_t)(h * g.D + d0 + k) << 4) + vperm(t)] = 0;
            }
        }
    }
}

}  // namespace tc
