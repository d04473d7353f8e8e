// Decode-step attention: one new token per query attends to everything its sequence already holds
// in the pool (the tables' tokens, the prompt's own suffix, the tokens generated so far) and to
// itself.  With one token, a KV head has only G rows (its group's query heads), so the work is
// reading K and V once: HBM-bound.  The prefill kernels serve this case too, but spend a 128-row
// tile and a chain of work-group barriers per key tile on it.
//
// Here the four waves of a work-group split the KEYS: wave w takes key tiles w, w+4, ... of the
// item's range, streams each straight into its own 32 KB of LDS (no work-group barrier in the
// loop: a wave waits only for its own loads), computes S^T = K . Q^T and O^T += V^T . P^T with the
// matrix cores exactly as the prefill kernels do (rows beyond G repeat row G-1 and are dropped)
// and keeps its own running maximum and sum.  At the end the four waves' (max, sum, O) are
// combined through LDS and the work-group writes one partial per row; a second kernel combines
// the key partitions of a query, adds the new token itself (its key and value come from k_new /
// v_new: one dot product and one scaled row per head) and writes the output.  The new token's
// K/V are appended to the pool by extra work-groups of the first launch, as in prefill.
#include "kv_append.h"
#include "lds_dma.h"
#include "tc_internal.h"

namespace tc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kDecHeadBlk = 4096;                    // one head's K (or V) in one block: 16 * 128 * 2
constexpr int kDecK = kAttnKeys * 256;               // K tile of a wave: 64 rows of 256 B, 16-byte chunks XOR-swizzled
constexpr int kDecWave = kDecK + 4 * kDecHeadBlk;    // + V tile: 32 KB per wave
constexpr int kDecBid = 4 * kDecWave + 256;          // block ids behind the four waves' tiles (+ alignment slack)
constexpr int kDecLds = kDecBid + kAttnMaxTiles * 4 * 4;
constexpr float kDecRescale = 8.f;

__global__ __launch_bounds__(256, 2) void decode_attn_bf16_kernel(Geom g, BatchDev b, AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    if ((int)blockIdx.x >= a.n_items) {                // extra work-groups: append the new tokens to the pool
        append_unit<true>(g, b, a.layer, (const char *)a.k_new, (const char *)a.v_new,
                          blockIdx.x - a.n_items, threadIdx.x);
        return;
    }
    const AttnItem it = a.items[blockIdx.x];
    if (it.q < 0) return;
    // the XOR addressing of the K tiles needs them 256-byte aligned
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds_raw;
    const uint32_t pad = (256u - (lds_base & 255u)) & 255u;
    char *lds = lds_raw + pad;
    const uint32_t lds0 = lds_base + pad;
    int32_t *s_bid = (int32_t *)(lds + kDecBid - 256);

    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, hh = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = g.G, P = it.P;
    const int n_tiles = it.tile_end - it.tile_begin;

    // block ids of the item's key range -> LDS (past the prefix: the last block, masked below)
    {
        const int last_pblk = max(((P + kBlockTokens - 1) >> 4) - 1, 0);
        const int32_t *bt = b.block_table + (int64_t)it.q * b.max_blocks;
        for (int idx = tid; idx < n_tiles * 4; idx += 256) s_bid[idx] = bt[min(it.tile_begin * 4 + idx, last_pblk)];
    }
    // Q^T fragments (B operand): lane (row r32, half hh) holds q[row][16*ks + 8*hh .. +8]
    const int head = it.kvh * G + min(r32, G - 1);
    bf16x8 qf[8];
    {
        const char *qp = (const char *)a.q + ((int64_t)it.cu * g.Hq + head) * 256 + hh * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = *(const bf16x8 *)(qp + ks * 32);
    }
    __syncthreads();                                    // block ids visible

    const char *pool_l = g.pool + (int64_t)a.layer * g.layer_stride + (int64_t)it.kvh * kDecHeadBlk;
    const int64_t bb = g.block_bytes;
    const uint32_t v_half = (uint32_t)(g.block_bytes >> 1);
    const uint32_t lds_w = lds0 + w * kDecWave;
    const float c = a.scale_log2;
    typedef const __attribute__((address_space(3))) bf16x8 *lds_frag;
    const uint32_t kb = lds_w + r32 * 256 + ((hh ^ (r32 & 15)) << 4);
    const uint32_t vb = lds_w + kDecK + r32 * 32 + hh * 16;

    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] = 0.f;
    float m_run = -INFINITY, l_lane = 0.f;

    // the four blocks of a tile: K as four 1 KB pieces of four rows each (chunk c of row r at
    // chunk position c ^ r), V verbatim; 16 load instructions per operand
    auto issue_k = [&](int t) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const char *src = pool_l + (int64_t)entry_bid(__builtin_amdgcn_readfirstlane(s_bid[t * 4 + j])) * bb;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rb = 4 * i + (lane >> 4);
                load_to_lds(lds_w + j * 4096 + i * 1024, src, rb * 256 + (((lane & 15) ^ rb) * 16));
            }
        }
    };
    auto issue_v = [&](int t) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const char *src = pool_l + (int64_t)entry_bid(__builtin_amdgcn_readfirstlane(s_bid[t * 4 + j])) * bb + v_half;
#pragma unroll
            for (int i = 0; i < 4; ++i) load_to_lds(lds_w + kDecK + j * 4096 + i * 1024, src + i * 1024, lane * 16);
        }
    };
    // Nobody but the wave reads its tile area, so the loop needs no barrier.  The loads run one
    // operand ahead: K of the next tile is requested as soon as this tile's K fragments sit in
    // registers, V likewise; loads complete in the order issued, so a wait that leaves the 16
    // younger ones outstanding has everything older in LDS.
    if (w < n_tiles) {
        issue_k(w);
        issue_v(w);
    }
    for (int t = w; t < n_tiles; t += 4) {
        const bool more = t + 4 < n_tiles;
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");      // K(t) has landed; V(t) may still be on its way

        // all operand fragments of a product are read from LDS before its matrix instructions start
        // (read one by one, each instruction would wait for its own LDS round trip)
        f32x16 sacc[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[mb][e] = 0.f;
        {
            bf16x8 kf[16];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) kf[2 * ks + mb] = *(lds_frag)(uintptr_t)((kb ^ (ks << 5)) + mb * 32 * 256);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");           // K area read out: free for the next tile
            if (more) issue_k(t + 4);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
                    sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[2 * ks + mb], qf[ks], sacc[mb], 0, 0, 0);
        }
        if (more) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");      // V(t) landed, K(t+4) outstanding
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        bf16x8 vf[16];                                 // V^T fragments: in registers before the softmax starts
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int db = 0; db < 4; ++db) vf[4 * kk + db] = *(lds_frag)(uintptr_t)(vb + kk * kDecHeadBlk + db * 1024);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");               // V area read out
        if (more) issue_v(t + 4);
        const int key0 = (it.tile_begin + t) * kAttnKeys;
        // positions that hold no key: beyond the end of the sequence, and the unused tail of a
        // table block read in place (its count rides in the block-table entry)
        const int4 e4 = *(const int4 *)&s_bid[t * 4];
        const int pad4 = entry_pad(e4.x) | (entry_pad(e4.y) << 8) | (entry_pad(e4.z) << 16) | (entry_pad(e4.w) << 24);
        if (pad4 != 0 || key0 + kAttnKeys > P) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int in_blk = 8 * ((e >> 2) & 1) + 4 * hh + (e & 3);
                    const int pad = (pad4 >> (8 * (2 * mb + (e >> 3)))) & 255;
                    const int key = key0 + 32 * mb + 8 * (e >> 2) + 4 * hh + (e & 3);
                    sacc[mb][e] = (key >= P || in_blk >= kBlockTokens - pad) ? -INFINITY : sacc[mb][e];
                }
        }
        float mx = sacc[0][0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sacc[0][e]);
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[1][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float mxs = mx * c;
        if (__any(mxs > m_run + kDecRescale)) {        // also taken while m_run is still -inf
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
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 pf;
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[e] = (__bf16)sacc[kk >> 1][8 * (kk & 1) + e];
#pragma unroll
            for (int db = 0; db < 4; ++db) o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[4 * kk + db], pf, o[db], 0, 0, 0);
        }
    }

    // ---- combine the four waves: each writes (max, sum) per row and O as [row][d] floats into its
    // own tile area (dead now), then every thread folds the four for a few (row, d)
    {
        float *wo = (float *)(lds + w * kDecWave);
        const float l_row = l_lane + __shfl_xor(l_lane, 32);
        if (r32 < G) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) wo[r32 * 128 + 32 * db + 8 * (e >> 2) + 4 * hh + (e & 3)] = o[db][e];
            if (hh == 0) { wo[32 * 128 + 2 * r32] = m_run; wo[32 * 128 + 2 * r32 + 1] = l_row; }
        }
    }
    __syncthreads();
    const int64_t n_rows = (int64_t)b.total_S * g.Hq;
    for (int idx = tid; idx < G * 128; idx += 256) {
        const int row = idx >> 7, d = idx & 127;
        float M = -INFINITY;
#pragma unroll
        for (int k = 0; k < 4; ++k) M = fmaxf(M, ((const float *)(lds + k * kDecWave))[32 * 128 + 2 * row]);
        float L = 0.f, acc = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float *wk = (const float *)(lds + k * kDecWave);
            const float mk = wk[32 * 128 + 2 * row];
            const float wgt = (mk == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mk - M);
            L += wgt * wk[32 * 128 + 2 * row + 1];
            acc += wgt * wk[row * 128 + d];
        }
        const int64_t slot = (int64_t)it.split * n_rows + (int64_t)it.cu * g.Hq + it.kvh * G + row;
        a.part_o[slot * 128 + d] = acc;
        if (d == 0) { a.part_ml[slot * 2] = M; a.part_ml[slot * 2 + 1] = L; }
    }
}

// One work-group of 128 threads per output row (token, head): combine the key partitions, add the
// new token itself, normalise, write bf16.
__global__ __launch_bounds__(128) void decode_finish_kernel(Geom g, BatchDev b, AttnArgs a, int max_splits)
{
    __shared__ float red[2];
    const int row = blockIdx.x, d = threadIdx.x;
    const int n = row / g.Hq, head = row - n * g.Hq, kvh = head / g.G;      // n: the token (queries may bring none)
    const int64_t n_rows = (int64_t)b.total_S * g.Hq;
    // Every load of the kernel is issued before the first use, so that the row costs one round
    // trip to memory: the query's partition count, the new token, and the first eight partitions'
    // partials (slots of partitions the query does not have exist in the buffer; they are loaded
    // and ignored).
    const int ns = b.splits_of_q[b.tok_q[n]];
    const unsigned short *q16 = (const unsigned short *)a.q + (int64_t)row * 128;
    const unsigned short *k16 = (const unsigned short *)a.k_new + ((int64_t)n * g.Hkv + kvh) * 128;
    const unsigned short *v16 = (const unsigned short *)a.v_new + ((int64_t)n * g.Hkv + kvh) * 128;
    const float qd = __uint_as_float((unsigned)q16[d] << 16), kd = __uint_as_float((unsigned)k16[d] << 16);
    const float vd = __uint_as_float((unsigned)v16[d] << 16);
    float2 ml[8];
    float po[8];
    auto fetch = [&](int s0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t slot = (int64_t)min(s0 + j, max_splits - 1) * n_rows + row;
            ml[j] = *(const float2 *)(a.part_ml + slot * 2);
            po[j] = a.part_o[slot * 128 + d];
        }
    };
    fetch(0);
    // score of the new token against itself
    float prod = qd * kd;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) prod += __shfl_xor(prod, off);
    if ((d & 63) == 0) red[d >> 6] = prod;
    __syncthreads();
    // running merge, started with the new token alone (weight 1 at its own score)
    float M = (red[0] + red[1]) * a.scale_log2, L = 1.f, acc = vd;
    for (int s0 = 0; s0 < ns; s0 += 8) {
        if (s0 > 0) fetch(s0);
        float Mc = M;
#pragma unroll
        for (int j = 0; j < 8; ++j) Mc = (s0 + j < ns) ? fmaxf(Mc, ml[j].x) : Mc;
        const float r = __builtin_amdgcn_exp2f(M - Mc);
        L *= r;
        acc *= r;
        M = Mc;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool live = s0 + j < ns && ml[j].x != -INFINITY;
            const float wgt = __builtin_amdgcn_exp2f(ml[j].x - M);
            L += live ? wgt * ml[j].y : 0.f;
            acc += live ? wgt * po[j] : 0.f;
        }
    }
    const __bf16 r = (__bf16)(acc / L);
    ((unsigned short *)a.out)[(int64_t)row * 128 + d] = *(const unsigned short *)&r;
}

hipError_t launch_decode_bf16(const Geom &g, const BatchDev &b, const AttnArgs &a, const Launch &L)
{
    if (a.n_items + a.n_append == 0) return hipSuccess;
    if (g.D != 128 || g.esize != 2 || g.G > 32) return hipErrorInvalidValue;
    static PerDeviceOnce configured;
    const hipError_t e = configured.run([] {
        return hipFuncSetAttribute((const void *)decode_attn_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kDecLds);
    });
    if (e != hipSuccess) return e;
    TC_LAUNCH(decode_attn_bf16_kernel, a.n_items + a.n_append, kDecLds, L, g, b, a);
    return hipGetLastError();
}

hipError_t launch_decode_finish(const Geom &g, const BatchDev &b, const AttnArgs &a, int max_splits, const Launch &L)
{
    const int n_rows = b.total_S * g.Hq;
    if (n_rows == 0) return hipSuccess;
    if (max_splits < 1) return hipErrorInvalidValue;
    hipExtLaunchKernelGGL(decode_finish_kernel, dim3(n_rows), dim3(128), 0, L.stream, L.start, L.stop, 0, g, b, a, max_splits);
    return hipGetLastError();
}

}  // namespace tc
