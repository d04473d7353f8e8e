// Suffix prefill attention on the gfx950 matrix cores: bf16 operands, fp32 accumulation.
//
// App. E.4 of the paper: only the uncached suffix is computed and it attends to all stitched
// table content (no mask) and causally to itself.  Because every row of one KV head - all
// suffix tokens times all G query heads of the group - reads the same keys and values, the
// rows are packed into one M dimension (row = token * G + head_in_group): a K/V tile is
// fetched once per KV head and shared by G*S rows, which is what makes the op compute-bound.
//
// Work-group: 4 waves, key tiles of 64 (= 4 pool blocks).  Each wave owns one or two blocks of 32
// rows (128 or 256 rows per work-group) and, per row block, computes the TRANSPOSED score tile S^T[key][row] = K . Q^T with v_mfma_f32_32x32x16_bf16, so
// that every lane holds scores of ONE row (column l%32 of the accumulator): row max, row sum and
// the output rescale need no cross-lane traffic except one exchange between lanes l and l^32.
// The exponentials, packed to bf16, are directly the B operand of O^T[d][row] += V^T . P^T; the
// pool stores V transposed inside a block with the token order the operand wants (kv_stitch.hip).
//
// Key tiles of a query: first the tiles of its stitched schema prefix, read from the pool through
// the block table (the last one ragged: keys >= P masked); then the tiles of its own suffix, read
// straight from k_new / v_new (token-major; V is transposed on its way into LDS) with the causal
// mask.  Because attention never reads the suffix from the pool, the append of the suffix to the
// pool is independent work: it runs in extra work-groups of the same launch.
//
// Memory pipeline: the work item carries the block ids of its first two tiles, the rest are
// fetched into LDS once; each iteration handles two key tiles, whose K/V travel global ->
// registers (issued a whole iteration ahead) -> two LDS buffers.  At batch 1 the kernel is
// latency-bound, so the depth of this pipeline and the length of the dependent-load chain at
// start-up are what matter.
//
// Split-KV: when a query is cut into key partitions, every work-group stores its partial
// (normalised O as fp16, max, sum) in accumulator-fragment order (512 B contiguous per wave and
// fragment) and a second kernel combines the partitions.  (Combining inside this kernel - last work-group to
// arrive folds the others in - was measured 3x slower: device-scope release/acquire on this chip
// writes back and invalidates the XCD's whole L2, which every work-group would do.)
#include "kv_append.h"
#include "tc_internal.h"

namespace tc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

constexpr int kKRow = 272;                       // LDS bytes per K row: 256 + 16 pad (conflict-free b128 reads)
constexpr int kHeadBlk = 4096;                   // bytes of one head's K (or V) in one block: 16 * 128 * 2
constexpr int kKTile = kAttnKeys * kKRow;        // 17408
constexpr int kVTile = 4 * kHeadBlk;             // 16384
constexpr int kStage = kKTile + kVTile;          // one LDS buffer
constexpr int kBidBytes = kAttnMaxTiles * 4 * 4; // block ids of the item's key range
constexpr int kLdsBytes = 2 * kStage + kBidBytes;
constexpr float kRescaleThresh = 8.f;            // log2 units: rescale O only when the max grew by more

// Per-lane state of RB row blocks (each row block = 32 rows of the wave, one row per lane pair).
template <int RB>
struct RowState {
    f32x16 o[RB][4];
    float m_run[RB], l_lane[RB];
};

// One key tile for RB row blocks: scores, online softmax, PV.  k_ld / v_ld already point at this
// lane's operands.  Every K and V fragment read from LDS feeds RB matrix instructions: with
// RB = 2 the LDS traffic per flop is half that of RB = 1, which is what the LDS (about 100 B per
// clock and CU, measured) can sustain next to the matrix cores.
template <int RB>
__device__ __forceinline__ void tile_math(RowState<RB> &st, const bf16x8 (&qf)[RB][8], const char *k_ld,
                                          const char *v_ld, int key0, const int (&limit)[RB],
                                          bool need_mask, int hh, float c)
{
    f32x16 sacc[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[rb][mb][e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            const bf16x8 ka = *(const bf16x8 *)(k_ld + mb * 32 * kKRow + ks * 32);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                sacc[rb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[rb][ks], sacc[rb][mb], 0, 0, 0);
        }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        if (need_mask) {                               // causal edge or ragged tail in this tile
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = key0 + 32 * mb + 8 * (e >> 2) + 4 * hh + (e & 3);
                    if (key > limit[rb]) sacc[rb][mb][e] = -INFINITY;
                }
        }
        float mx = sacc[rb][0][0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sacc[rb][0][e]);
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[rb][1][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float mxs = mx * c;
        if (__any(mxs > st.m_run[rb] + kRescaleThresh)) {   // also taken while m_run is still -inf
            const float m_new = fmaxf(st.m_run[rb], mxs);
            const float alpha = (st.m_run[rb] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.m_run[rb] - m_new);
            st.l_lane[rb] *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) st.o[rb][db][e] *= alpha;
            st.m_run[rb] = m_new;
        }
        const float neg_m = (st.m_run[rb] == -INFINITY) ? 0.f : -st.m_run[rb];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sacc[rb][mb][e], c, neg_m));
                sacc[rb][mb][e] = p;
                st.l_lane[rb] += p;
            }
    }
    // O^T[d][row] += V^T[d][key] P^T[key][row]: four 16-key groups (one pool block each)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        bf16x8 pf[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[rb][e] = (__bf16)sacc[rb][kk >> 1][8 * (kk & 1) + e];
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const bf16x8 va = *(const bf16x8 *)(v_ld + kk * kHeadBlk + db * 32 * 32);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                st.o[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pf[rb], st.o[rb][db], 0, 0, 0);
        }
    }
}

// RB = row blocks per wave: the work-group covers 128 * RB rows.  RB = 1 runs two work-groups per
// CU (small problems: more, smaller work items); RB = 2 one per CU with twice the work per LDS byte.
template <int RB>
__global__ __launch_bounds__(256, RB == 1 ? 2 : 1) void attn_bf16_kernel(Geom g, BatchDev b, AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    int32_t *s_bid = (int32_t *)(lds + 2 * kStage);

    if ((int)blockIdx.x >= a.n_items) {                // extra work-groups: append the suffix to the pool
        append_unit<true>(g, b, a.layer, (const char *)a.k_new, (const char *)a.v_new,
                          blockIdx.x - a.n_items, threadIdx.x);
        return;
    }
    const AttnItem it = a.items[blockIdx.x];
    if (it.q < 0) return;                              // padding item (uniform for the work-group)
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r32 = lane & 31, hh = lane >> 5;
    const int G = g.G, P = it.P, S = it.S;
    const int npt = (P + kAttnKeys - 1) >> 6;          // prefix tiles; suffix tiles follow
    const int last_pblk = max(((P + kBlockTokens - 1) >> 4) - 1, 0);
    const int m_rows = S * G;
    const int wave_row0 = it.m0 + w * 32 * RB;
    bool valid[RB];
    int s_tok[RB], head[RB], limit[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row_m = wave_row0 + rb * 32 + r32;
        valid[rb] = row_m < m_rows;
        const int rm = valid[rb] ? row_m : m_rows - 1;
        s_tok[rb] = rm / G;
        head[rb] = it.kvh * G + (rm - s_tok[rb] * G);
        limit[rb] = s_tok[rb];                         // last visible suffix key of this row
    }
    const int wave_stok_min = min(wave_row0, m_rows - 1) / G;
    const int n_tiles = it.tile_end - it.tile_begin, last = n_tiles - 1;
    // Addresses are (uniform 64-bit base) + (32-bit per-thread offset), so that the loads take their
    // base from scalar registers and no 64-bit address arithmetic or registers are spent per load.
    const char *pool_l = g.pool + (int64_t)a.layer * g.layer_stride + (int64_t)it.kvh * kHeadBlk;
    const uint32_t v_half = (uint32_t)(g.block_bytes >> 1);
    const int64_t bb = g.block_bytes;
    const uint32_t t_off = tid * 16;
    // suffix rows: this thread's 16-byte chunk of the row of token (16*i + tid/16) of a suffix tile
    const uint32_t new_row = (uint32_t)g.Hkv * 256;
    const char *kn_s = (const char *)a.k_new + (int64_t)it.cu * new_row + it.kvh * 256;
    const char *vn_s = (const char *)a.v_new + (int64_t)it.cu * new_row + it.kvh * 256;
    const uint32_t c_off = (tid & 15) * 16;
    const int t16 = tid >> 4;
    const int tv = tid & 15;                           // V of suffix tiles: token within the block,
    const uint32_t cv_off = (tid >> 4) * 16;           // and 16-byte chunk of its row

    // Q^T fragments (B operand): lane (row r32, half hh) holds q[row][16*ks + 8*hh .. +8].
    // Issued before any K/V load: vector loads return in order, so once the first K/V tile has
    // arrived these have too, and no wait on them is left inside the tile loop (a wait there
    // would drain the K/V prefetches every iteration).
    bf16x8 qf[RB][8];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const char *qp = (const char *)a.q + ((int64_t)(it.cu + s_tok[rb]) * g.Hq + head[rb]) * 256 + hh * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[rb][ks] = *(const bf16x8 *)(qp + ks * 32);
    }
    // named prefetch registers (arrays of uint4 end up in scratch): set A and set B
    uint4 ka0, ka1, ka2, ka3, va0, va1, va2, va3;
    uint4 kb0, kb1, kb2, kb3, vb0, vb1, vb2, vb3;
#define TC_LD(kx, vx, bid_)                                                                    \
    {                                                                                          \
        const char *src = pool_l + (int64_t)__builtin_amdgcn_readfirstlane(bid_) * bb;        \
        kx = *(const uint4 *)(src + t_off);                                                    \
        vx = *(const uint4 *)(src + (v_half + t_off));                                         \
    }
    // suffix tile: K chunk of row (tok_ + tid/16), like a pool block; V chunk of row (tok_ + tid%16),
    // eight d-values starting at 8 * (tid/16) - the assignment the transposing LDS store wants
#define TC_LD_NEW(kx, vx, tok_)                                                                \
    {                                                                                          \
        kx = *(const uint4 *)(kn_s + ((uint32_t)min((tok_) + t16, S - 1) * new_row + c_off));  \
        vx = *(const uint4 *)(vn_s + ((uint32_t)min((tok_) + tv, S - 1) * new_row + cv_off));  \
    }
    // Every prefetch is issued unconditionally, eight loads per tile whatever its kind (past the
    // end of the range the tile index is clamped and the data never used): with loads under a
    // condition the compiler cannot count how many are outstanding and falls back to waiting for
    // all of them, which empties the pipeline.
    // First two tiles: block ids come with the item.
    if (it.tile_begin < npt) {
        TC_LD(ka0, va0, it.bid[0]) TC_LD(ka1, va1, it.bid[1]) TC_LD(ka2, va2, it.bid[2]) TC_LD(ka3, va3, it.bid[3])
    } else {
        const int t0_ = (it.tile_begin - npt) * kAttnKeys;
        TC_LD_NEW(ka0, va0, t0_) TC_LD_NEW(ka1, va1, t0_ + 16) TC_LD_NEW(ka2, va2, t0_ + 32) TC_LD_NEW(ka3, va3, t0_ + 48)
    }
    if (it.tile_begin + 1 < npt) {
        TC_LD(kb0, vb0, it.bid[4]) TC_LD(kb1, vb1, it.bid[5]) TC_LD(kb2, vb2, it.bid[6]) TC_LD(kb3, vb3, it.bid[7])
    } else {
        const int t0_ = max(it.tile_begin + 1 - npt, 0) * kAttnKeys;
        TC_LD_NEW(kb0, vb0, t0_) TC_LD_NEW(kb1, vb1, t0_ + 16) TC_LD_NEW(kb2, vb2, t0_ + 32) TC_LD_NEW(kb3, vb3, t0_ + 48)
    }
    // block ids of the whole key range -> LDS
    {
        const int32_t *bt = b.block_table + (int64_t)it.q * b.max_blocks;
        for (int idx = tid; idx < n_tiles * 4; idx += 256)     // past the prefix: a valid block, never used
            s_bid[idx] = bt[min(it.tile_begin * 4 + idx, last_pblk)];
    }
    RowState<RB> st;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) st.o[rb][db][e] = 0.f;
        st.m_run[rb] = -INFINITY;
        st.l_lane[rb] = 0.f;
    }
    const float c = a.scale_log2;

    char *k_st = lds + (tid >> 4) * kKRow + (tid & 15) * 16;        // + stage * kStage
    char *v_st = lds + kKTile + tid * 16;
    const char *k_ld = lds + r32 * kKRow + hh * 16;
    const char *v_ld = lds + kKTile + r32 * 32 + hh * 16;
    // V of a suffix tile arrives token-major and must land as [d][token] (the pool's transposed
    // block layout, which the PV operand reads).  Lanes l and l^1 hold the same eight d-values of
    // two adjacent tokens: they swap registers (DPP), the even lane packs the even d of both tokens
    // into dwords, the odd lane the odd d, so each lane issues 4 dword stores per chunk.
    const int odd_tok = tv & 1;
    const uint32_t vt_off = (uint32_t)(tid >> 4) * 256 + odd_tok * 32 + (vperm(tv) >> 1) * 4;
#define TC_ST_VT(vd_, v_)                                                                         \
    {                                                                                             \
        const unsigned u_[4] = {(v_).x, (v_).y, (v_).z, (v_).w};                                  \
        _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_) {                                        \
            const unsigned p_ = (unsigned)__builtin_amdgcn_update_dpp(0, (int)u_[j_], 0xB1, 0xF, 0xF, false); \
            const unsigned w_ = odd_tok ? ((p_ >> 16) | (u_[j_] & 0xffff0000u))                   \
                                        : ((u_[j_] & 0xffffu) | (p_ << 16));                      \
            *(unsigned *)((vd_) + vt_off + j_ * 64) = w_;                                         \
        }                                                                                         \
    }
#define TC_ST(stage_, is_new_, k0_, k1_, k2_, k3_, v0_, v1_, v2_, v3_)                           \
    {                                                                                             \
        char *kd = k_st + (stage_) * kStage, *vd = v_st + (stage_) * kStage;                      \
        *(uint4 *)(kd) = k0_;                                                                     \
        *(uint4 *)(kd + 16 * kKRow) = k1_;                                                        \
        *(uint4 *)(kd + 32 * kKRow) = k2_;                                                        \
        *(uint4 *)(kd + 48 * kKRow) = k3_;                                                        \
        if (!(is_new_)) {                                                                         \
            *(uint4 *)(vd) = v0_;                                                                 \
            *(uint4 *)(vd + kHeadBlk) = v1_;                                                      \
            *(uint4 *)(vd + 2 * kHeadBlk) = v2_;                                                  \
            *(uint4 *)(vd + 3 * kHeadBlk) = v3_;                                                  \
        } else {                                                                                  \
            char *vt = lds + (stage_) * kStage + kKTile;                                          \
            TC_ST_VT(vt, v0_) TC_ST_VT(vt + kHeadBlk, v1_)                                        \
            TC_ST_VT(vt + 2 * kHeadBlk, v2_) TC_ST_VT(vt + 3 * kHeadBlk, v3_)                     \
        }                                                                                         \
    }
#define TC_LD_TILE(r_, k0_, k1_, k2_, k3_, v0_, v1_, v2_, v3_)                                    \
    {                                                                                             \
        const int rr_ = (r_);                                                                     \
        if (it.tile_begin + rr_ < npt) {                                                          \
            const int32_t *bp = s_bid + rr_ * 4;                                                  \
            TC_LD(k0_, v0_, bp[0]) TC_LD(k1_, v1_, bp[1]) TC_LD(k2_, v2_, bp[2]) TC_LD(k3_, v3_, bp[3]) \
        } else {                                                                                  \
            const int t0_ = (it.tile_begin + rr_ - npt) * kAttnKeys;                              \
            TC_LD_NEW(k0_, v0_, t0_) TC_LD_NEW(k1_, v1_, t0_ + 16)                                \
            TC_LD_NEW(k2_, v2_, t0_ + 32) TC_LD_NEW(k3_, v3_, t0_ + 48)                           \
        }                                                                                         \
    }
#define TC_LD_TILE_A(r_) TC_LD_TILE(r_, ka0, ka1, ka2, ka3, va0, va1, va2, va3)
#define TC_LD_TILE_B(r_) TC_LD_TILE(r_, kb0, kb1, kb2, kb3, vb0, vb1, vb2, vb3)
    // prefix tile: keys count from 0 and the last valid one is P-1; suffix tile: keys count from the
    // first suffix token and row r sees those up to its own token
#define TC_MATH(r_, stage_)                                                                       \
    {                                                                                             \
        const int tt_ = it.tile_begin + (r_);                                                     \
        const bool pre_ = tt_ < npt;                                                              \
        const int key0 = (pre_ ? tt_ : tt_ - npt) * kAttnKeys;                                    \
        int lim_[RB];                                                                             \
        _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) lim_[rb] = pre_ ? P - 1 : limit[rb];    \
        tile_math<RB>(st, qf, k_ld + (stage_) * kStage, v_ld + (stage_) * kStage, key0, lim_,     \
                      key0 + kAttnKeys - 1 > (pre_ ? P - 1 : wave_stok_min), hh, c);              \
    }

    // Two key tiles (128 keys) per iteration: their K/V are loaded into the two register sets
    // one whole iteration before they are stored to LDS, so the only wait the loads ever need is
    // "all outstanding", at a point where a full iteration of math has covered their latency.
    for (int r = 0; r < n_tiles; r += 2) {
        const bool new_a = it.tile_begin + min(r, last) >= npt, new_b = it.tile_begin + min(r + 1, last) >= npt;
        __syncthreads();                               // both LDS stages free (s_bid visible on the first pass)
        TC_ST(0, new_a, ka0, ka1, ka2, ka3, va0, va1, va2, va3)
        TC_ST(1, new_b, kb0, kb1, kb2, kb3, vb0, vb1, vb2, vb3)
        __syncthreads();
        TC_LD_TILE_A(min(r + 2, last))
        TC_LD_TILE_B(min(r + 3, last))
        TC_MATH(r, 0)
        if (r + 1 < n_tiles) TC_MATH(r + 1, 1)
    }
#undef TC_LD
#undef TC_LD_NEW
#undef TC_ST
#undef TC_ST_VT
#undef TC_LD_TILE
#undef TC_LD_TILE_A
#undef TC_LD_TILE_B
#undef TC_MATH

#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const float l = st.l_lane[rb] + __shfl_xor(st.l_lane[rb], 32);
        if (it.n_splits > 1) {
            // partial in accumulator-fragment order, normalised and stored as fp16 (outputs of a
            // softmax average are bounded by max|v|, so fp16's 11-bit mantissa costs ~3e-5 here and
            // halves the partial traffic, the largest cost of a split launch): 512 B contiguous per
            // (row block, db, q4); a group's slot holds 4 * RB row blocks of 32 rows
            const int64_t slot = (int64_t)it.split * it.n_groups + it.group;
            const int blk = w * RB + rb;
            const float inv = l > 0.f ? 1.f / l : 0.f;
            f16x4 *po = (f16x4 *)a.part_o + ((slot * (4 * RB) + blk) * 16) * 64 + lane;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (_Float16)(st.o[rb][db][4 * q4 + e] * inv);
                    po[(db * 4 + q4) * 64] = v;
                }
            if (hh == 0)
                ((float2 *)a.part_ml)[(slot * (4 * RB) + blk) * 32 + r32] = make_float2(st.m_run[rb], l);
            continue;
        }
        if (!valid[rb]) continue;
        const int64_t row = (int64_t)(it.cu + s_tok[rb]) * g.Hq + head[rb];
        const float inv = 1.f / l;
        char *op = (char *)a.out + row * 256 + hh * 8;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (__bf16)(st.o[rb][db][4 * q4 + e] * inv);
                *(bf16x4 *)(op + (32 * db + 8 * q4) * 2) = v;
            }
    }
}

// Combine the partitions of split queries.  One thread per 4 values of a group's accumulator
// fragment: index = ((group * n_rb + row_block) * 16 + fragment) * 64 + lane, the order the
// attention kernel stored it in, so loads are fully coalesced.  With reference maxima m_s, sums
// l_s and normalised partial outputs O_s:  out = sum_s w_s O_s / sum_s w_s,  w_s = 2^(m_s - M) l_s.
__global__ __launch_bounds__(256) void merge_bf16_kernel(Geom g, AttnArgs a, const MergeGroup *groups,
                                                         int n_groups, int n_rb)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int lane = idx & 63, frag = (idx >> 6) & 15, gb = idx >> 10;
    const int group = gb / n_rb, blk = gb - group * n_rb;
    if (group >= n_groups) return;
    const MergeGroup mg = groups[group];
    if (mg.n_splits <= 1) return;                      // written directly by the attention kernel
    const int r32 = lane & 31, hh = lane >> 5;
    const int row_m = mg.m0 + blk * 32 + r32;
    if (row_m >= mg.S * g.G) return;
    // partitions in chunks of 8: all loads of a chunk are issued before anything waits on them
    float M = -INFINITY, l = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    const int64_t stride = (int64_t)n_groups * n_rb;          // (group, block) slots per partition
    const int64_t gb0 = (int64_t)group * n_rb + blk;
    for (int s0 = 0; s0 < mg.n_splits; s0 += 8) {
        f16x4 v[8];
        float2 ml[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int s = min(s0 + k, mg.n_splits - 1);
            const int64_t sb = (int64_t)s * stride + gb0;
            v[k] = ((const f16x4 *)a.part_o)[(sb * 16 + frag) * 64 + lane];
            ml[k] = ((const float2 *)a.part_ml)[sb * 32 + r32];
        }
        float Mc = M;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (s0 + k < mg.n_splits) Mc = fmaxf(Mc, ml[k].x);
        const float resc = (M == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(M - Mc);   // earlier chunks -> new reference
        l *= resc; acc.x *= resc; acc.y *= resc; acc.z *= resc; acc.w *= resc;
        M = Mc;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            if (s0 + k >= mg.n_splits) continue;
            const float wgt = (ml[k].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ml[k].x - M) * ml[k].y;
            l += wgt;
            acc.x = fmaf(wgt, (float)v[k][0], acc.x); acc.y = fmaf(wgt, (float)v[k][1], acc.y);
            acc.z = fmaf(wgt, (float)v[k][2], acc.z); acc.w = fmaf(wgt, (float)v[k][3], acc.w);
        }
    }
    const float inv = 1.f / l;
    const int s_tok = row_m / g.G;
    const int head = mg.kvh * g.G + (row_m - s_tok * g.G);
    const int db = frag >> 2, q4 = frag & 3;
    bf16x4 o;
    o[0] = (__bf16)(acc.x * inv); o[1] = (__bf16)(acc.y * inv);
    o[2] = (__bf16)(acc.z * inv); o[3] = (__bf16)(acc.w * inv);
    *(bf16x4 *)((char *)a.out + ((int64_t)(mg.cu + s_tok) * g.Hq + head) * 256 + (32 * db + 8 * q4 + 4 * hh) * 2) = o;
}

template <int RB>
static hipError_t launch_attn_rb(const Geom &g, const BatchDev &b, const AttnArgs &a, const Launch &L)
{
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void *)attn_bf16_kernel<RB>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    TC_LAUNCH(attn_bf16_kernel<RB>, a.n_items + a.n_append, kLdsBytes, L, g, b, a);
    return hipGetLastError();
}

hipError_t launch_attn_bf16(const Geom &g, const BatchDev &b, const AttnArgs &a, int row_blocks, const Launch &L)
{
    if (a.n_items + a.n_append == 0) return hipSuccess;
    if (g.D != 128 || g.esize != 2) return hipErrorInvalidValue;
    if (row_blocks == 1) return launch_attn_rb<1>(g, b, a, L);
    if (row_blocks == 2) return launch_attn_rb<2>(g, b, a, L);
    return hipErrorInvalidValue;
}

hipError_t launch_merge_bf16(const Geom &g, const AttnArgs &a, const MergeGroup *groups, int n_groups,
                             int row_blocks, const Launch &L)
{
    if (n_groups == 0) return hipSuccess;
    const int n_rb = 4 * row_blocks;                   // 32-row blocks per group
    TC_LAUNCH(merge_bf16_kernel, n_groups * n_rb * 4, 0, L, g, a, groups, n_groups, n_rb);
    return hipGetLastError();
}

}  // namespace tc
