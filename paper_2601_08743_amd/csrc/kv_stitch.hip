// KV stitch (gather of table segments into sequence blocks), suffix append and
// read-back kernels.  All three are pure byte movement: HBM-bound, 128-bit accesses.
//
// Sequence-block layout in one layer (private to the library):
//   K half: [Hkv][16 tokens][D]                        (token rows, as the QK^T operand wants them)
//   V half: fp32: [Hkv][16 tokens][D]
//           bf16: [Hkv][D][16 tokens], token t stored at position vperm(t) so that the two
//                 8-token groups a PV matrix-core operand needs are 16 contiguous bytes.
#include <algorithm>

#include "kv_append.h"
#include "tc_internal.h"

namespace tc {

__device__ __forceinline__ uint4 keep_if(uint4 v, bool keep)        // v, or zeros
{
    v.x = keep ? v.x : 0u;
    v.y = keep ? v.y : 0u;
    v.z = keep ? v.z : 0u;
    v.w = keep ? v.w : 0u;
    return v;
}

// Copy of one block: token rows [t][h][d] at k_src / v_src + src_off[t] (-1: no such token, zeros)
// -> the block's K half [h][t][d] at dst and its V half at vdst (through `lds`, [16][row_bytes / 16]
// chunks, where 2-byte elements are transposed per head).
//
// A missing token is loaded from offset 0 (always valid) and the value replaced: written as
// "offset >= 0 ? load : zero" the compiler selects between the global address and the address of a
// zero it first stores to scratch memory - 32 bytes of stores per thread, a quarter on top of the
// block's own bytes.  The loads of a pass (kCopyBatch chunks of K and of V per thread) are all
// issued before the first store, so that a thread has 128 bytes in flight instead of 16.
constexpr int kCopyBatch = 4;

// K chunk c of the destination, in address order: consecutive threads write consecutive 16 bytes
// (a wave covers 1 KB of one head: four token rows), and read 256-byte pieces of four source rows.
__device__ __forceinline__ uint4 load_k_chunk(const Geom &g, const char *k_src, const int64_t *src_off, int c, bool &ok)
{
    const int cph = g.head_bytes >> 4;
    const int ht = c / cph, dc = c - ht * cph;
    const int h = ht / kBlockTokens, t = ht - h * kBlockTokens;
    const int64_t so = src_off[t];
    ok = so >= 0;
    return *(const uint4 *)(k_src + (ok ? so : 0) + ((int64_t)(h * cph + dc) << 4));
}
// V chunk c in source order (token t, chunk w of its row)
__device__ __forceinline__ uint4 load_v_chunk(const Geom &g, const char *v_src, const int64_t *src_off, int c, bool &ok)
{
    const int cpr = g.row_bytes >> 4;
    const int t = c / cpr, w = c - t * cpr;
    const int64_t so = src_off[t];
    ok = so >= 0;
    return *(const uint4 *)(v_src + (ok ? so : 0) + ((int64_t)w << 4));
}
// where V chunk c goes when it is not transposed: [h][t][d]
__device__ __forceinline__ int64_t v_plain_offset(const Geom &g, int c)
{
    const int cpr = g.row_bytes >> 4, cph = g.head_bytes >> 4;
    const int t = c / cpr, w = c - t * cpr;
    const int h = w / cph, dc = w - h * cph;
    return (int64_t)(h * kBlockTokens + t) * g.head_bytes + (dc << 4);
}

// second half of the transposing path: out chunk oc = (h, d, half): 8 tokens of one (h, d)
// t_first > 0: tokens below t_first keep what the block already holds: `old` brings the block's
// chunks (chunk tid + 256 k in old[k]), read by the caller before anything else so that the read is
// not one more round trip at the end; they are merged and written back.
constexpr int kOldChunks = 8;                  // covers Hkv * D * 2 <= 2048 chunks; beyond that the chunk is read here
__device__ __forceinline__ void store_v_transposed(const Geom &g, const uint4 *lds, char *vdst, int tid, int t_first = 0,
                                                   const uint4 *old_pre = nullptr)
{
    const unsigned short *l16 = (const unsigned short *)lds;
    const int row_elems = g.row_bytes >> 1;
    const int n_out = g.Hkv * g.D * 2;
    for (int k = 0; tid + 256 * k < n_out; ++k) {
        const int oc = tid + 256 * k;
        const int half = oc & 1;
        const int hd = oc >> 1;                // h * D + d
        uint4 old = make_uint4(0, 0, 0, 0);
        if (t_first > 0) {
            if (old_pre && k < kOldChunks) {
                // (selected, not indexed, so that the array stays in registers)
#pragma unroll
                for (int q = 0; q < kOldChunks; ++q) if (q == k) old = old_pre[q];
            } else {
                old = *(const uint4 *)(vdst + ((int64_t)oc << 4));
            }
        }
        const unsigned o32[4] = {old.x, old.y, old.z, old.w};
        unsigned short e[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int t = (k & 3) | ((k & 4) << 1) | (half << 2);
            const unsigned short fresh = l16[t * row_elems + hd];
            e[k] = t >= t_first ? fresh : (unsigned short)(o32[k >> 1] >> (16 * (k & 1)));
        }
        uint4 v;
        v.x = e[0] | ((unsigned)e[1] << 16);
        v.y = e[2] | ((unsigned)e[3] << 16);
        v.z = e[4] | ((unsigned)e[5] << 16);
        v.w = e[6] | ((unsigned)e[7] << 16);
        *(uint4 *)(vdst + ((int64_t)oc << 4)) = v;
    }
}

// The values alone (the re-encoding stitch turns the keys itself).
template <bool kTransposeV>
__device__ __forceinline__ void copy_block_v(const Geom &g, const char *v_src, const int64_t *src_off, char *vdst,
                                             uint4 *lds, int tid)
{
    const int n_chunks = kBlockTokens * (g.row_bytes >> 4);
    for (int c0 = tid; c0 < n_chunks; c0 += 256 * kCopyBatch) {
        uint4 v[kCopyBatch];
        bool ok[kCopyBatch];
#pragma unroll
        for (int j = 0; j < kCopyBatch; ++j) v[j] = load_v_chunk(g, v_src, src_off, min(c0 + 256 * j, n_chunks - 1), ok[j]);
#pragma unroll
        for (int j = 0; j < kCopyBatch; ++j) {
            const int c = c0 + 256 * j;
            if (c >= n_chunks) continue;
            if (kTransposeV) lds[c] = keep_if(v[j], ok[j]);
            else *(uint4 *)(vdst + v_plain_offset(g, c)) = keep_if(v[j], ok[j]);
        }
    }
    if (kTransposeV) {
        __syncthreads();
        store_v_transposed(g, lds, vdst, tid);
    }
}

// Keys and values of one block together.
template <bool kTransposeV>
__device__ __forceinline__ void copy_block_kv(const Geom &g, const char *k_src, const char *v_src, const int64_t *src_off,
                                              char *dst, char *vdst, uint4 *lds, int tid, int t_first = 0)
{
    const int n_chunks = kBlockTokens * (g.row_bytes >> 4);
    const int cpr = g.row_bytes >> 4, cph = g.head_bytes >> 4;
    uint4 old_v[kOldChunks];
    if (kTransposeV && t_first > 0) {              // the shared block's values, on their way while the rows are fetched
        const int n_out = g.Hkv * g.D * 2;
#pragma unroll
        for (int k = 0; k < kOldChunks; ++k)
            old_v[k] = *(const uint4 *)(vdst + ((int64_t)min(tid + 256 * k, n_out - 1) << 4));
    }
    for (int c0 = tid; c0 < n_chunks; c0 += 256 * kCopyBatch) {
        uint4 kk[kCopyBatch], vv[kCopyBatch];
        bool kok[kCopyBatch], vok[kCopyBatch];
#pragma unroll
        for (int j = 0; j < kCopyBatch; ++j) kk[j] = load_k_chunk(g, k_src, src_off, min(c0 + 256 * j, n_chunks - 1), kok[j]);
#pragma unroll
        for (int j = 0; j < kCopyBatch; ++j) vv[j] = load_v_chunk(g, v_src, src_off, min(c0 + 256 * j, n_chunks - 1), vok[j]);
#pragma unroll
        for (int j = 0; j < kCopyBatch; ++j) {
            const int c = c0 + 256 * j;
            // (K chunk c belongs to token (c / cph) % 16, V chunk c to token c / cpr)
            if (c < n_chunks && (c / cph) % kBlockTokens >= t_first) *(uint4 *)(dst + ((int64_t)c << 4)) = keep_if(kk[j], kok[j]);
        }
#pragma unroll
        for (int j = 0; j < kCopyBatch; ++j) {
            const int c = c0 + 256 * j;
            if (c >= n_chunks) continue;
            if (kTransposeV) lds[c] = keep_if(vv[j], vok[j]);
            else if (c / cpr >= t_first) *(uint4 *)(vdst + v_plain_offset(g, c)) = keep_if(vv[j], vok[j]);
        }
    }
    if (kTransposeV) {
        __syncthreads();
        store_v_transposed(g, lds, vdst, tid, t_first, old_v);
    }
}


// ------------------------------------------------------------------------------------ stitch
// Paper Sec. 4.1.2: the matched tables' KV caches are concatenated in match order.
// One work-group per (destination block, layer).
//
// kRope (Sec. 4.1.1, last paragraph): the stored keys carry no positional encoding and get it
// here, while they are copied, from their global position in the concatenated sequence: rotary
// encoding in the half-split convention, pair (i, i + D/2) of every head turned by
// pos * theta^(-2i/D).  The turn is taken as a fraction of a revolution in fp64 (pos times a
// per-frequency constant the host computed in fp64; only the fraction matters), so positions of
// tens of thousands lose nothing; sine and cosine of that fraction (fp32 storage: accurate library
// routine; bf16 storage: the hardware instructions, whose ~1e-6 error is far below the result's
// rounding) and the rotation itself are fp32, the result is rounded once to the storage type.
// V is copied unchanged.
template <bool kTransposeV, bool kRope>
__global__ __launch_bounds__(256) void stitch_kernel(Geom g, BatchDev b, int l0)
{
    extern __shared__ uint4 lds[];                 // the rotation table, then (transposing path) V rows [16][row_bytes/16]
    __shared__ int64_t src_off[kBlockTokens];
    const StitchBlk blk = b.stitch_blk[blockIdx.x];
    const int layer = l0 + blockIdx.y;
    const int tid = threadIdx.x;
    if (tid < kBlockTokens) {
        const int p = blk.p0 + tid;
        int64_t off = -1;
        if (p < b.prefix_len[blk.q]) {
            int s = blk.seg;
            while (p >= b.seg_start[s] + b.seg_len[s]) ++s;
            off = (int64_t)b.seg_slot[s] * g.slot_bytes +
                  ((int64_t)layer * b.seg_len[s] + (p - b.seg_start[s])) * g.row_bytes;
        }
        src_off[tid] = off;
    }
    __syncthreads();
    const char *layer_base = g.tab_base;             // source rows: table slots
    char *dst = g.pool + (int64_t)layer * g.layer_stride + (int64_t)blk.phys * g.block_bytes;
    const int cpr = g.row_bytes >> 4;              // 16-byte chunks per token row
    const int cph = g.head_bytes >> 4;             // ... per head
    const int n_chunks = kBlockTokens * cpr;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    if (!kRope) {
        copy_block_kv<kTransposeV>(g, layer_base, layer_base + (g.slot_bytes >> 1), src_off, dst, dst + (g.block_bytes >> 1), lds, tid);
        return;
    } else {
        // one unit = the two 16-byte chunks of a head row that hold elements i and i + D/2.  The
        // loads of a pass of kUnits units per thread are issued first; the rotation table is built
        // while they are in flight.
        const int half_d = g.D >> 1;
        const int half_c = cph >> 1;
        const int n_units = kBlockTokens * g.Hkv * half_c;
        constexpr int kElems = kTransposeV ? 8 : 4;                 // elements per chunk: bf16 or fp32
        constexpr int kUnits = 4;
        float2 *cs = (float2 *)lds;             // shares the V staging area: a barrier separates the two uses
        const int64_t pos_base = (int64_t)b.rope_pos0[blk.q] + blk.p0;
        bool table_ready = false;
        for (int u0 = tid; u0 < n_units; u0 += 256 * kUnits) {
            uint4 va[kUnits], vb[kUnits];
#pragma unroll
            for (int j = 0; j < kUnits; ++j) {
                const int u = u0 + 256 * j;
                va[j] = zero;
                vb[j] = zero;
                if (u < n_units) {
                    const int t = u / (g.Hkv * half_c), r = u - t * (g.Hkv * half_c);
                    const int h = r / half_c, cc = r - h * half_c;
                    const int64_t so = src_off[t];
                    if (so >= 0) {
                        const char *src = layer_base + so + ((int64_t)(h * cph + cc) << 4);
                        va[j] = *(const uint4 *)src;
                        vb[j] = *(const uint4 *)(src + (half_c << 4));
                    }
                }
            }
            if (!table_ready) {
                // (cos, sin) of every (token of the block, frequency): [16][D/2] float2
                for (int idx = tid; idx < kBlockTokens * half_d; idx += 256) {
                    const int t = idx / half_d, i = idx - t * half_d;
                    const double turns = (double)(pos_base + t) * b.rope_rev_freq[i];
                    const float frac = (float)(turns - floor(turns));      // [0, 1) of a revolution
                    float sn, c;
                    if (kTransposeV) {                                      // bf16 results: the hardware's sine / cosine
                        sn = __builtin_amdgcn_sinf(frac);                   // (argument in revolutions, ~1e-6 absolute)
                        c = __builtin_amdgcn_cosf(frac);
                    } else {
                        sincospif(2.0f * frac, &sn, &c);
                    }
                    cs[idx] = make_float2(c, sn);
                }
                __syncthreads();
                table_ready = true;
            }
#pragma unroll
            for (int j = 0; j < kUnits; ++j) {
                const int u = u0 + 256 * j;
                if (u >= n_units) continue;
                const int t = u / (g.Hkv * half_c), r = u - t * (g.Hkv * half_c);
                const int h = r / half_c, cc = r - h * half_c;
                const float2 *csr = cs + t * half_d + cc * kElems;
                uint4 oa, ob;
                if (kTransposeV) {                                      // bf16 storage
                    const unsigned ua[4] = {va[j].x, va[j].y, va[j].z, va[j].w}, ub[4] = {vb[j].x, vb[j].y, vb[j].z, vb[j].w};
                    unsigned ra[4], rb[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        float xa[2] = {__uint_as_float(ua[k] << 16), __uint_as_float(ua[k] & 0xffff0000u)};
                        float xb[2] = {__uint_as_float(ub[k] << 16), __uint_as_float(ub[k] & 0xffff0000u)};
                        unsigned short pa[2], pb[2];
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            const float2 w = csr[2 * k + e];
                            const __bf16 na = (__bf16)(xa[e] * w.x - xb[e] * w.y);
                            const __bf16 nb = (__bf16)(xb[e] * w.x + xa[e] * w.y);
                            pa[e] = *(const unsigned short *)&na;
                            pb[e] = *(const unsigned short *)&nb;
                        }
                        ra[k] = pa[0] | ((unsigned)pa[1] << 16);
                        rb[k] = pb[0] | ((unsigned)pb[1] << 16);
                    }
                    oa = make_uint4(ra[0], ra[1], ra[2], ra[3]);
                    ob = make_uint4(rb[0], rb[1], rb[2], rb[3]);
                } else {                                                // fp32 storage
                    const float xa[4] = {__uint_as_float(va[j].x), __uint_as_float(va[j].y), __uint_as_float(va[j].z), __uint_as_float(va[j].w)};
                    const float xb[4] = {__uint_as_float(vb[j].x), __uint_as_float(vb[j].y), __uint_as_float(vb[j].z), __uint_as_float(vb[j].w)};
                    float na[4], nb[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float2 w = csr[e];
                        na[e] = xa[e] * w.x - xb[e] * w.y;
                        nb[e] = xb[e] * w.x + xa[e] * w.y;
                    }
                    oa = make_uint4(__float_as_uint(na[0]), __float_as_uint(na[1]), __float_as_uint(na[2]), __float_as_uint(na[3]));
                    ob = make_uint4(__float_as_uint(nb[0]), __float_as_uint(nb[1]), __float_as_uint(nb[2]), __float_as_uint(nb[3]));
                }
                char *d = dst + (int64_t)(h * kBlockTokens + t) * g.head_bytes + (cc << 4);
                *(uint4 *)d = oa;
                *(uint4 *)(d + (half_c << 4)) = ob;
            }
        }
        __syncthreads();                        // the rotation table is dead: the V staging may overwrite it
    }
    copy_block_v<kTransposeV>(g, layer_base + (g.slot_bytes >> 1), src_off, dst + (g.block_bytes >> 1), lds, tid);
}

// ------------------------------------------------------------------------------------ format
// A table's KV as registered (token rows, all layers: K part then V part) -> the blocks of its
// slot, in the sequence-block layout, the unused tail of its last block zero-filled (keys and
// values), so that an attention launch can read the slot's blocks as if they were part of a
// stitched sequence.  One work-group per (block of the table, layer).  `raw` holds the K part at
// offset 0 and the V part at `v_part`; layer l of either starts n_tokens * l rows in.
template <bool kTransposeV>
__global__ __launch_bounds__(256) void format_kernel(Geom g, const char *raw, int64_t v_part, int n_tokens,
                                                     int first_block, int l0)
{
    extern __shared__ uint4 lds[];
    __shared__ int64_t src_off[kBlockTokens];
    const int layer = l0 + blockIdx.y;
    const int tid = threadIdx.x;
    if (tid < kBlockTokens) {
        const int tok = blockIdx.x * kBlockTokens + tid;
        src_off[tid] = tok < n_tokens ? ((int64_t)layer * n_tokens + tok) * g.row_bytes : -1;
    }
    __syncthreads();
    char *dst = g.pool + (int64_t)layer * g.layer_stride + (int64_t)(first_block + blockIdx.x) * g.block_bytes;
    copy_block_kv<kTransposeV>(g, raw, raw + v_part, src_off, dst, dst + (g.block_bytes >> 1), lds, tid);
}

hipError_t launch_format(const Geom &g, const void *raw, int64_t v_part, int n_tokens, int first_block, int l0,
                         int l1, const Launch &L)
{
    if (n_tokens <= 0 || l1 <= l0) return hipSuccess;
    dim3 grid((n_tokens + kBlockTokens - 1) / kBlockTokens, l1 - l0);
    if (g.esize == 2)
        TC_LAUNCH(format_kernel<true>, grid, kBlockTokens * g.row_bytes, L, g, (const char *)raw, v_part, n_tokens,
                  first_block, l0);
    else
        TC_LAUNCH(format_kernel<false>, grid, 0, L, g, (const char *)raw, v_part, n_tokens, first_block, l0);
    return hipGetLastError();
}

hipError_t launch_stitch(const Geom &g, const BatchDev &b, int l0, int l1, bool rope, const Launch &L)
{
    if (b.n_stitch_blk == 0 || l1 <= l0) return hipSuccess;
    dim3 grid(b.n_stitch_blk, l1 - l0);
    const size_t cs_bytes = rope ? (size_t)kBlockTokens * (g.D >> 1) * sizeof(float2) : 0;
    const size_t v_bytes = (size_t)kBlockTokens * g.row_bytes;
    if (rope && (!b.rope_pos0 || !b.rope_rev_freq || (g.D & 1) || ((g.head_bytes >> 4) & 1))) return hipErrorInvalidValue;
    if (g.esize == 2) {
        if (rope) TC_LAUNCH((stitch_kernel<true, true>), grid, std::max(v_bytes, cs_bytes), L, g, b, l0);
        else TC_LAUNCH((stitch_kernel<true, false>), grid, kBlockTokens * g.row_bytes, L, g, b, l0);
    } else {
        if (rope) TC_LAUNCH((stitch_kernel<false, true>), grid, cs_bytes, L, g, b, l0);
        else TC_LAUNCH((stitch_kernel<false, false>), grid, 0, L, g, b, l0);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ append
// Stand-alone launch of the append units (fp32 path), one work-group per unit.
template <bool kTransposeV>
__global__ __launch_bounds__(256) void append_kernel(Geom g, BatchDev b, int layer,
                                                     const char *k_new, const char *v_new)
{
    append_unit<kTransposeV>(g, b, layer, k_new, v_new, blockIdx.x, threadIdx.x);
}

// Append by blocks, for launches that must have the suffix in the pool before attention starts:
// one work-group per sequence block that holds suffix tokens.  A block that lies wholly behind the
// prefix is written like a stitched block (rows of k_new / v_new as the source, zeros behind the
// end of the sequence); in the one block a query may share with its prefix the prefix tokens stay
// (keys: their rows are skipped; transposed values: 16 bytes read, merged, written back).
template <bool kTransposeV>
__global__ __launch_bounds__(256) void append_blocks_kernel(Geom g, BatchDev b, int layer,
                                                            const char *k_new, const char *v_new)
{
    extern __shared__ uint4 lds[];
    __shared__ int64_t src_off[kBlockTokens];
    const int tid = threadIdx.x;
    // which query, which of its blocks: the queries' block counts are fetched 256 at a time (one
    // round trip), then every thread walks them in LDS
    __shared__ int s_P[256], s_S[256], s_cu[256];
    int rem = blockIdx.x, i = -1, P = 0, S = 0, cu = 0;
    for (int i0 = 0; i0 < b.B && i < 0; i0 += 256) {
        if (i0 + tid < b.B) {
            const int c0 = b.cu_seqlens[i0 + tid];
            s_P[tid] = b.prefix_len[i0 + tid];
            s_S[tid] = b.cu_seqlens[i0 + tid + 1] - c0;
            s_cu[tid] = c0;
        }
        __syncthreads();
        const int m = min(256, b.B - i0);
        for (int j = 0; j < m; ++j) {
            const int Pq = s_P[j], Sq = s_S[j];
            const int nb = Sq > 0 ? ((Pq + Sq + kBlockTokens - 1) >> 4) - (Pq >> 4) : 0;
            if (rem < nb) { i = i0 + j; P = Pq; S = Sq; cu = s_cu[j]; break; }
            rem -= nb;
        }
        __syncthreads();
    }
    if (i < 0) return;
    // token t of the block is suffix token p0 + t - P (none before the prefix ends or behind the
    // sequence's end: the former keep what the stitch wrote, the latter become zeros)
    const int blk = (P >> 4) + rem, p0 = blk * kBlockTokens;
    const int t_first = max(P - p0, 0);
    if (tid < kBlockTokens) {
        const int pos = p0 + tid;
        src_off[tid] = pos >= P && pos < P + S ? (int64_t)(cu + pos - P) * g.row_bytes : -1;
    }
    __syncthreads();
    const int phys = entry_bid(b.block_table[(int64_t)i * b.max_blocks + blk]);
    char *dst = g.pool + (int64_t)layer * g.layer_stride + (int64_t)phys * g.block_bytes;
    copy_block_kv<kTransposeV>(g, k_new, v_new, src_off, dst, dst + (g.block_bytes >> 1), lds, tid, t_first);
}

hipError_t launch_append_blocks(const Geom &g, const BatchDev &b, int layer, const void *k_new, const void *v_new,
                                int n_blocks, const Launch &L)
{
    if (n_blocks == 0) return hipSuccess;
    if (g.esize == 2)
        TC_LAUNCH(append_blocks_kernel<true>, n_blocks, kBlockTokens * g.row_bytes, L, g, b, layer, (const char *)k_new, (const char *)v_new);
    else
        TC_LAUNCH(append_blocks_kernel<false>, n_blocks, 0, L, g, b, layer, (const char *)k_new, (const char *)v_new);
    return hipGetLastError();
}

hipError_t launch_append(const Geom &g, const BatchDev &b, int layer, const void *k_new,
                         const void *v_new, const Launch &L)
{
    const int n = b.total_S + b.B;
    if (n == 0) return hipSuccess;
    if (g.esize == 2)
        TC_LAUNCH(append_kernel<true>, n, 0, L, g, b, layer, (const char *)k_new, (const char *)v_new);
    else
        TC_LAUNCH(append_kernel<false>, n, 0, L, g, b, layer, (const char *)k_new, (const char *)v_new);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ read-back
// Undo the block layout: token-major [n_tokens][Hkv][D] for K and V.  One work-group per block.
template <bool kTransposeV>
__global__ __launch_bounds__(256) void readback_kernel(Geom g, int layer, const int32_t *blocks,
                                                       int n_tokens, char *k_out, char *v_out)
{
    const int tid = threadIdx.x;
    const int jb = blockIdx.x;
    const int phys = blocks[jb];
    const char *kd = g.pool + (int64_t)layer * g.layer_stride + (int64_t)phys * g.block_bytes;
    const char *vd = kd + (g.block_bytes >> 1);
    const int cpr = g.row_bytes >> 4, cph = g.head_bytes >> 4;
    for (int c = tid; c < kBlockTokens * cpr; c += 256) {
        const int t = c / cpr, w = c - t * cpr;
        const int p = jb * kBlockTokens + t;
        if (p >= n_tokens) continue;
        const int h = w / cph, dc = w - h * cph;
        *(uint4 *)(k_out + (int64_t)p * g.row_bytes + (w << 4)) =
            *(const uint4 *)(kd + (int64_t)(h * kBlockTokens + t) * g.head_bytes + (dc << 4));
        if (!kTransposeV) {
            *(uint4 *)(v_out + (int64_t)p * g.row_bytes + (w << 4)) =
                *(const uint4 *)(vd + (int64_t)(h * kBlockTokens + t) * g.head_bytes + (dc << 4));
        } else {
            const unsigned short *v16 = (const unsigned short *)vd;
            unsigned short *o16 = (unsigned short *)(v_out + (int64_t)p * g.row_bytes + (w << 4));
            const int d0 = dc << 3;
#pragma unroll
            for (int k = 0; k < 8; ++k) o16[k] = v16[((int64_t)(h * g.D + d0 + k) << 4) + vperm(t)];
        }
    }
}

hipError_t launch_readback(const Geom &g, int layer, const int32_t *blocks_dev, int n_tokens,
                           void *k_out_dev, void *v_out_dev, hipStream_t s)
{
    if (n_tokens <= 0) return hipSuccess;
    const int nb = (n_tokens + kBlockTokens - 1) / kBlockTokens;
    if (g.esize == 2)
        readback_kernel<true><<<nb, 256, 0, s>>>(g, layer, blocks_dev, n_tokens, (char *)k_out_dev,
                                                 (char *)v_out_dev);
    else
        readback_kernel<false><<<nb, 256, 0, s>>>(g, layer, blocks_dev, n_tokens, (char *)k_out_dev,
                                                  (char *)v_out_dev);
    return hipGetLastError();
}

}  // namespace tc
