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
#include "lds_dma.h"
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

// Matrix instructions written as inline assembly with their accumulator in ordinary registers
// (defined with the pipelined path below, where the reason is given).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void mfma_first(f32x16 &acc, const bf16x8 &a, const bf16x8 &b);
__device__ __forceinline__ void mfma_v(f32x16 &acc, const bf16x8 &a, const bf16x8 &b);

// One key tile for RB row blocks: scores, online softmax, PV.  k_ld / v_ld already point at this
// lane's operands.  Every K and V fragment read from LDS feeds RB matrix instructions: with
// RB = 2 the LDS traffic per flop is half that of RB = 1, which is what the LDS (about 100 B per
// clock and CU, measured) can sustain next to the matrix cores.
// kAsmScores (the kernel that may use 512 registers per wave): left to itself the compiler puts the
// score accumulators into accumulation registers there and copies all 32 of them out, one by
// one, for the softmax.  The QK matrix instructions are therefore issued as inline assembly with
// the accumulators in ordinary registers, and a fence holds the 12 wait states a matrix result
// needs before a vector instruction may read it (the compiler does not see those instructions'
// latency).  (O stays with the compiler here: it keeps O in ordinary registers between tiles and
// copies it into accumulation registers and back around every tile's PV; issuing the PV
// instructions as assembly with an accumulation-register operand did not stop that, and gave
// wrong results besides - left alone.)
template <int RB, bool kAsmScores>
__device__ __forceinline__ void tile_math(RowState<RB> &st, const bf16x8 (&qf)[RB][8], const char *k_ld,
                                          const char *v_ld, int key0, const int (&limit)[RB],
                                          bool need_mask, uint32_t pads, int hh, float c)
{
    f32x16 sacc[RB][2];
    if (!kAsmScores) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) sacc[rb][mb][e] = 0.f;
    }
    // The operand fragments run two reads ahead of the matrix instruction that consumes them (a ring
    // of three): read one by one in front of its instruction, every fragment costs a full LDS round
    // trip during which the wave issues nothing.
    {
        bf16x8 kf[3];
#define TC_KFRAG(j) (*(const bf16x8 *)(k_ld + ((j) & 1) * 32 * kKRow + ((j) >> 1) * 32))
        kf[0] = TC_KFRAG(0);
        kf[1] = TC_KFRAG(1);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int ks = j >> 1, mb = j & 1;
            if (j + 2 < 16) kf[(j + 2) % 3] = TC_KFRAG(j + 2);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                if (!kAsmScores) sacc[rb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j % 3], qf[rb][ks], sacc[rb][mb], 0, 0, 0);
                else if (ks == 0) mfma_first(sacc[rb][mb], kf[j % 3], qf[rb][ks]);
                else mfma_v(sacc[rb][mb], kf[j % 3], qf[rb][ks]);
            }
        }
#undef TC_KFRAG
    }
    if (kAsmScores) {
        static_assert(!kAsmScores || RB == 1, "one row block per wave");
        asm volatile("s_nop 11" : "+v"(sacc[0][0]), "+v"(sacc[0][1]));
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        if (need_mask) {                               // causal edge, ragged tail or unused block tails in this tile
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = key0 + 32 * mb + 8 * (e >> 2) + 4 * hh + (e & 3);
                    // position inside its 16-token block, and that block's unused tail (4 bits per block)
                    const int t = 8 * ((e >> 2) & 1) + 4 * hh + (e & 3);
                    const int used = 16 - (int)((pads >> (4 * (2 * mb + (e >> 3)))) & 15u);
                    const bool dead = (key > limit[rb]) | (t >= used);     // a select, not a branch
                    sacc[rb][mb][e] = dead ? -INFINITY : sacc[rb][mb][e];
                }
        }
        float mx = sacc[rb][0][0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sacc[rb][0][e]);
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[rb][1][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float mxs = mx * c;
        if (__builtin_expect(__any(mxs > st.m_run[rb] + kRescaleThresh), 0)) {   // rare; also taken while m_run is still -inf
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
    {
        bf16x8 vf[3];
#define TC_VFRAG(j) (*(const bf16x8 *)(v_ld + ((j) >> 2) * kHeadBlk + ((j) & 3) * 32 * 32))
        vf[0] = TC_VFRAG(0);
        vf[1] = TC_VFRAG(1);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 pf[RB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[rb][e] = (__bf16)sacc[rb][kk >> 1][8 * (kk & 1) + e];
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const int j = 4 * kk + db;
                if (j + 2 < 16) vf[(j + 2) % 3] = TC_VFRAG(j + 2);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    st.o[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[j % 3], pf[rb], st.o[rb][db], 0, 0, 0);
            }
        }
#undef TC_VFRAG
    }
}

// Geometry of one work item as every part of the kernel sees it.
template <int RB>
struct ItemRows {
    bool valid[RB];
    int s_tok[RB], head[RB], limit[RB];
    int wave_row0, wave_stok_min, m_rows;
};

template <int RB>
__device__ __forceinline__ void item_rows(ItemRows<RB> &ir, const Geom &g, const AttnItem &it, int w, int r32)
{
    ir.m_rows = it.S * g.G;
    ir.wave_row0 = it.m0 + w * 32 * RB;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row_m = ir.wave_row0 + rb * 32 + r32;
        ir.valid[rb] = row_m < ir.m_rows;
        const int rm = ir.valid[rb] ? row_m : ir.m_rows - 1;
        ir.s_tok[rb] = rm / g.G;
        ir.head[rb] = it.kvh * g.G + (rm - ir.s_tok[rb] * g.G);
        ir.limit[rb] = ir.s_tok[rb];                   // last visible suffix key of this row
    }
    ir.wave_stok_min = min(ir.wave_row0, ir.m_rows - 1) / g.G;
}

// Q^T fragments (B operand): lane (row r32, half hh) holds q[row][16*ks + 8*hh .. +8].
template <int RB>
__device__ __forceinline__ void load_q(bf16x8 (&qf)[RB][8], const Geom &g, const AttnArgs &a, const AttnItem &it,
                                       const ItemRows<RB> &ir, int hh)
{
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const char *qp = (const char *)a.q + ((int64_t)(it.cu + ir.s_tok[rb]) * g.Hq + ir.head[rb]) * 256 + hh * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[rb][ks] = *(const bf16x8 *)(qp + ks * 32);
    }
}

// Block ids of the item's key range -> LDS (past the prefix: a valid block, never used).
__device__ __forceinline__ void fill_bids(int32_t *s_bid, const BatchDev &b, const AttnItem &it, int tid)
{
    const int last_pblk = max(((it.P + kBlockTokens - 1) >> 4) - 1, 0);
    const int n_tiles = it.tile_end - it.tile_begin;
    const int32_t *bt = b.block_table + (int64_t)it.q * b.max_blocks;
    for (int idx = tid; idx < n_tiles * 4; idx += 256) s_bid[idx] = bt[min(it.tile_begin * 4 + idx, last_pblk)];
}

// The general key-tile loop: tiles [r0, n_tiles) of the item, any mix of prefix tiles (pool, through
// the block ids in LDS), the ragged last prefix tile and causal suffix tiles (k_new / v_new).
// K/V travel global -> registers (issued a whole iteration = two tiles ahead) -> two LDS buffers of
// kStage bytes at the start of `lds`.  With r0 == 0 the first two tiles take their block ids from the
// item, so their loads do not wait for the block-id table; `do_fill` then fills that table here,
// after the loads are on their way.
template <int RB, bool kAsmScores>
__device__ __forceinline__ void tile_loop(RowState<RB> &st, const bf16x8 (&qf)[RB][8], const Geom &g,
                                          const BatchDev &b, const AttnArgs &a, const AttnItem &it,
                                          const ItemRows<RB> &ir, char *lds, int32_t *s_bid, int r0, bool do_fill,
                                          int tid)
{
    const int lane = tid & 63, r32 = lane & 31, hh = lane >> 5;
    const int P = it.P, S = it.S;
    const int npt = (P + kAttnKeys - 1) >> 6;          // prefix tiles; suffix tiles follow
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

    // named prefetch registers (arrays of uint4 end up in scratch): set A and set B
    uint4 ka0, ka1, ka2, ka3, va0, va1, va2, va3;
    uint4 kb0, kb1, kb2, kb3, vb0, vb1, vb2, vb3;
#define TC_LD(kx, vx, bid_)                                                                    \
    {                                                                                          \
        const char *src = pool_l + (int64_t)entry_bid(__builtin_amdgcn_readfirstlane(bid_)) * bb; \
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
    // Every prefetch is issued unconditionally, eight loads per tile whatever its kind (past the
    // end of the range the tile index is clamped and the data never used): with loads under a
    // condition the compiler cannot count how many are outstanding and falls back to waiting for
    // all of them, which empties the pipeline.
    if (r0 == 0) {
        // first two tiles: block ids come with the item
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
    } else {
        TC_LD_TILE_A(min(r0, last))
        TC_LD_TILE_B(min(r0 + 1, last))
    }
    if (do_fill) fill_bids(s_bid, b, it, tid);
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
    // prefix tile: keys count from 0 and the last valid one is P-1; suffix tile: keys count from the
    // first suffix token and row r sees those up to its own token
#define TC_MATH(r_, stage_)                                                                       \
    {                                                                                             \
        const int tt_ = it.tile_begin + (r_);                                                     \
        const bool pre_ = tt_ < npt;                                                              \
        const int key0 = (pre_ ? tt_ : tt_ - npt) * kAttnKeys;                                    \
        int lim_[RB];                                                                             \
        _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) lim_[rb] = pre_ ? P - 1 : ir.limit[rb]; \
        uint32_t pads_ = 0;                                                                       \
        if (pre_) {                                                                               \
            const int4 e4_ = *(const int4 *)(s_bid + (r_) * 4);                                   \
            pads_ = (uint32_t)entry_pad(e4_.x) | ((uint32_t)entry_pad(e4_.y) << 4) |              \
                    ((uint32_t)entry_pad(e4_.z) << 8) | ((uint32_t)entry_pad(e4_.w) << 12);       \
            pads_ = __builtin_amdgcn_readfirstlane(pads_);                                        \
        }                                                                                         \
        tile_math<RB, kAsmScores>(st, qf, k_ld + (stage_) * kStage, v_ld + (stage_) * kStage, key0, lim_, \
                      pads_ != 0 || key0 + kAttnKeys - 1 > (pre_ ? P - 1 : ir.wave_stok_min),     \
                      pads_, hh, c);                                                              \
    }

    // Two key tiles (128 keys) per iteration: their K/V are loaded into the two register sets
    // one whole iteration before they are stored to LDS, so the only wait the loads ever need is
    // "all outstanding", at a point where a full iteration of math has covered their latency.
    for (int r = r0; r < n_tiles; r += 2) {
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
}

// Final normalisation and store: the output rows, or (split queries) this partition's partial.
template <int RB>
__device__ __forceinline__ void store_rows(const RowState<RB> &st, const Geom &g, const AttnArgs &a,
                                           const AttnItem &it, const ItemRows<RB> &ir, int w, int lane)
{
    const int r32 = lane & 31, hh = lane >> 5;
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
                    __builtin_nontemporal_store(v, &po[(db * 4 + q4) * 64]);
                }
            if (hh == 0)
            {
                typedef float f32x2 __attribute__((ext_vector_type(2)));
                f32x2 ml;
                ml[0] = st.m_run[rb];
                ml[1] = l;
                __builtin_nontemporal_store(ml, &((f32x2 *)a.part_ml)[(slot * (4 * RB) + blk) * 32 + r32]);
            }
            continue;
        }
        if (!ir.valid[rb]) continue;
        const int64_t row = (int64_t)(it.cu + ir.s_tok[rb]) * g.Hq + ir.head[rb];
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

template <int RB>
__device__ __forceinline__ void reset_rows(RowState<RB> &st)
{
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) st.o[rb][db][e] = 0.f;
        st.m_run[rb] = -INFINITY;
        st.l_lane[rb] = 0.f;
    }
}

// The plain kernel: the general tile loop over the whole key range.  RB = row blocks per wave: the
// work-group covers 128 * RB rows; RB = 2 runs one work-group per CU with twice the work per LDS byte.
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
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    ItemRows<RB> ir;
    item_rows<RB>(ir, g, it, w, lane & 31);
    // Q is issued before any K/V load: vector loads return in order, so once the first K/V tile has
    // arrived these have too, and no wait on them is left inside the tile loop (a wait there
    // would drain the K/V prefetches every iteration).
    bf16x8 qf[RB][8];
    load_q<RB>(qf, g, a, it, ir, lane >> 5);
    RowState<RB> st;
    reset_rows<RB>(st);
    tile_loop<RB, false>(st, qf, g, b, a, it, ir, lds, s_bid, 0, true, tid);
    store_rows<RB>(st, g, a, it, ir, w, lane);
}

// ------------------------------------------------------------------------------------------------
// The pipelined path for runs of full, unmasked prefix tiles (the bulk of a long schema prefix).
//
// Three things distinguish it from the general loop:
//  * A fixed softmax reference per row (the maximum over the first 32 keys of the run) instead of
//    a running maximum: p = 2^(s*c - ref) needs no per-tile maximum and O is never rescaled, so
//    only matrix instructions touch O.  Any finite reference gives the same quotient O / l; what can
//    go wrong is overflow when later scores exceed the reference by ~2^100, which is detected from l
//    after the run and answered by redoing the item in the general loop (running maximum).
//  * A three-stage software pipeline inside every wave: step s issues the matrix instructions of
//    QK^T for tile s+1 and of PV for tile s-1 while the vector unit turns the scores of tile s into
//    weights.  One matrix instruction, one LDS operand read (three slots ahead) and the fused
//    multiply-add / exp2 / add / pack of one score - each belonging to a different score, so none waits
//    on the one before - make a "slot"; a step is 32 slots in a fixed order.
//  * K/V tiles go from global memory straight into LDS (global_load_lds_dwordx4: lane l's 16 bytes
//    land at M0 + 16 l), which frees the 64 registers the general loop stages two tiles in and lets
//    loads run four tiles ahead.  Four K buffers + four V buffers (128 KB) hold them; K rows are 256 B
//    with the 16-byte chunk index XORed with (row & 15) - each lane picks the global chunk that
//    belongs at its LDS position - so the operand reads are bank-conflict free without padding.
//
// Timeline (tiles of the run are 0 .. n-1):  prime: QK(0), reference, weights of its first 32 keys;
// step s = 0 .. n: QK(s+1) | weights of tile s keys 32..63 and tile s+1 keys 0..31 | PV(s-1).
// Between steps: wait for the tiles the next step reads, barrier, issue the loads that reuse the
// buffers the finished step released: K(s+5) into K(s+1)'s, V(s+3) into V(s-1)'s.
constexpr int kFastKTile = kAttnKeys * 256;               // 16 KB, swizzled rows
constexpr int kFastBufs = 4;
constexpr int kFastV = kFastBufs * kFastKTile;            // V buffers follow the K buffers
constexpr int kFastBid = kFastV + kFastBufs * kVTile;     // block ids of the item's key range (up to kPipeMaxTiles tiles)
constexpr int kLdsBytesPipe = kFastBid + kPipeMaxTiles * 4 * 4;
static_assert(kLdsBytesPipe <= 160 * 1024 && 2 * kStage <= kFastBid, "LDS layout");
// Shorter runs take the general loop: they are mostly the pipeline's fill and drain (two tiles were
// measured slower than the general loop, three within a few percent of it either way).
// History of this limit.  An earlier build returned launch-dependent rows for runs of exactly three
// tiles and the limit was raised to four before the cause was known.  The cause, found since by
// building that source again with the limit at three (wrong in 117 of 120 fresh contexts): under
// register pressure the compiler kept a Q fragment in accumulation registers and reloaded it
// (v_accvgpr_read) directly in front of a hand-placed QK matrix instruction.  A matrix instruction
// must not read a register a vector instruction wrote less than two wait states earlier; the
// compiler keeps that rule for its own matrix instructions and cannot for inline assembly.  Five
// idle slots in front of every hand-placed matrix instruction made that build right (0 of 120); so
// did naming the score registers in the step's closing fence (which this source does), because it
// changed the allocation and the reload went away.  That the rule holds in the emitted code -
// no vector write to a source of a hand-placed matrix instruction in the two wait states before
// it - is now checked by tests/test_kernel_schedule.py, which fails on that earlier source; with
// it, this source runs three-tile runs correctly when the limit is lowered (160 + 200 fresh
// contexts, bits equal across launches).
constexpr int kFastMinTiles = 4;

#define TC_SB() __builtin_amdgcn_sched_barrier(0)

struct FastState {
    f32x16 S[4];        // scores / weights in stream order: even tile keys 32..63, odd tile keys 0..31,
                        // odd tile keys 32..63, even tile keys 0..31
    u32x4 pE[4], pO[4]; // packed bf16 weights of the last even / odd tile, one register set per 16 keys
    float l, nm;        // this lane's part of the row sum; minus the reference (log2 units)
};

// The instructions of the pipelined steps are written out one by one.  The compiler still allocates
// the registers and inserts the waits for the LDS reads, but it neither reorders these instructions
// nor chooses their register classes, and both matter here:
//  * the kernel runs one work-group per CU (LDS), so a wave may use 512 registers, but only 256 of
//    them are ordinary VGPRs; the others (AGPRs) can only be accumulators.  O is touched by nothing
//    but matrix instructions in these steps, so it lives there ("a" below) and leaves the VGPRs to
//    the scores, weights, Q and operand fragments ("v").  Left to itself the compiler puts every
//    accumulator of such a kernel, the scores included, into AGPRs and copies them out one by one.
//  * a matrix instruction's result must not be read by a vector instruction for 11 cycles after
//    issue, and the hardware does not interlock this: the fixed order below keeps every such pair
//    three or more slots (> 100 cycles) apart.
__device__ __forceinline__ void mfma_first(f32x16 &acc, const bf16x8 &a, const bf16x8 &b)     // acc = a b
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_v(f32x16 &acc, const bf16x8 &a, const bf16x8 &b)         // acc += a b
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_a(f32x16 &acc, const bf16x8 &a, const u32x4 &b)          // same, AGPR accumulator
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void v_scale(float &x, float c, float nm)                          // x = x c + nm
{
    asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x) : "s"(c), "v"(nm));
}
__device__ __forceinline__ void v_exp2(float &x) { asm volatile("v_exp_f32 %0, %0" : "+v"(x)); }
__device__ __forceinline__ void v_acc(float &l, float x) { asm volatile("v_add_f32 %0, %0, %1" : "+v"(l) : "v"(x)); }
__device__ __forceinline__ void v_pack(uint32_t &d, float lo, float hi)
{
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(d) : "v"(lo), "v"(hi));
}

// The compiler does not know how long a matrix instruction written as inline assembly takes, and it
// is free to put its own register copies of O (moves between accumulation registers where two
// paths join, copies in and out of them) right next to one.  These two fences pin O down: each
// names all of O as an operand, so every copy the compiler makes lands before `o_fence_in` or after
// `step_fence_out`.  A matrix result must not be read for 11 cycles after issue (the compiler's own
// figure for this instruction): the closing fence sits right behind the step's last matrix
// instruction and holds 12.  After the opening fence the first matrix instruction that reads O
// comes more than ten instructions later, which covers the 2 cycles a freshly written register needs.
__device__ __forceinline__ void o_fence_in(f32x16 (&o)[4])
{
    asm volatile("" : "+a"(o[0]), "+a"(o[1]), "+a"(o[2]), "+a"(o[3]));
}
// The closing fence also names the score registers (ordinary VGPRs, written by the QK matrix
// instructions): no compiler-made copy of them may follow the step's last matrix instructions
// closely either.
__device__ __forceinline__ void step_fence_out(f32x16 (&o)[4], f32x16 (&S)[4])
{
    asm volatile("s_nop 11" : "+a"(o[0]), "+a"(o[1]), "+a"(o[2]), "+a"(o[3]),
                              "+v"(S[0]), "+v"(S[1]), "+v"(S[2]), "+v"(S[3]));
}

// One step.  PAR = parity of s.  kb / vb: this lane's LDS read addresses for K(s+1) / V(s-1); the
// K chunk of k-step ks sits at kb ^ (ks << 5) (the XOR swizzle; bits 5..7 of kb hold the lane's key).
// QK: tile s+1 exists, PV: tile s-1 exists - compile-time, because a run-time test per matrix
// instruction costs 12 % of a step.  They switch only the matrix instructions: the vector
// work runs unconditionally (on stale registers where a tile does not exist: finite, and never
// used); the row sum collects the weights of tile s and of tile s+1 separately (l_cur, l_nxt) and
// the caller adds each only if its tile exists.
template <int PAR, bool QK, bool PV>
__device__ __forceinline__ void fast_step(FastState &fs, f32x16 (&o)[4], const bf16x8 (&qf)[8], uint32_t kb,
                                          uint32_t vb, float c, float &l_cur, float &l_nxt)
{
    u32x4 (&Pcur)[4] = PAR == 0 ? fs.pE : fs.pO;       // weights of tile s (parity PAR)
    u32x4 (&Pnxt)[4] = PAR == 0 ? fs.pO : fs.pE;       // weights of tiles s-1 and s+1
    const float nm = fs.nm;
    float lc = 0.f, ln = 0.f;
    bf16x8 fr[4];
    typedef const __attribute__((address_space(3))) bf16x8 *lds_frag;
    // LDS address of the A operand of slot j: even j = QK op j/2 (32-key half mb = op/8, k-step ks =
    // op%8); odd j = PV op (j-1)/2 (16-key group kk = op/4, 32 d-values db = op%4)
#define TC_OPADDR(j) ((((j) & 1) == 0) ? (kb ^ ((((j) >> 1) & 7) << 5)) + (((j) >> 4) * 32 * 256)             \
                                      : vb + ((((j) >> 1) >> 2) * kHeadBlk + (((j) >> 1) & 3) * 1024))
#define TC_OPLOAD(j) if ((((j) & 1) == 0) ? QK : PV) fr[(j) & 3] = *(lds_frag)(uintptr_t)(TC_OPADDR(j));
    if (PV) o_fence_in(o);
    TC_OPLOAD(0) TC_OPLOAD(1) TC_OPLOAD(2)
    // stream position x of this step: 0..15 -> S[2 PAR] (tile s, keys 32..63), 16..31 -> S[2 PAR + 1]
    // (tile s+1, keys 0..31); negative: the previous step's positions 32 + x (tile s, keys 0..31)
#define TC_SREG(x) fs.S[(x) >= 16 ? 2 * PAR + 1 : (x) >= 0 ? 2 * PAR : 3 - 2 * PAR][(x) & 15]
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        if (j + 3 < 32) TC_OPLOAD(j + 3)
        // vector work, one stage for each of four different scores
        {
            const int xf = j - 2, xe = j - 3, xa = j - 4, xc = j - 5;
            if (xf < 32) { float t = TC_SREG(xf); v_scale(t, c, nm); TC_SREG(xf) = t; }
            if (xe < 32) { float t = TC_SREG(xe); v_exp2(t); TC_SREG(xe) = t; }
            if (xa < 32) {
                if (xa >= 16) v_acc(ln, TC_SREG(xa));
                else v_acc(lc, TC_SREG(xa));
            }
            if (xc & 1) {
                // pack scores xc-1, xc: element y of their tile -> dword y/2 of that tile's weights
                const int y = xc >= 16 ? xc - 16 : 16 + xc;       // xc < 16: tile s (keys 0..31 if xc < 0)
                const int d = (xc >= 16 || xc < 0) ? (y >> 1) : 8 + (xc >> 1);
                uint32_t pk;
                v_pack(pk, TC_SREG(xc - 1), TC_SREG(xc));
                if (xc >= 16) Pnxt[d >> 2][d & 3] = pk;
                else Pcur[d >> 2][d & 3] = pk;
            }
        }
        if ((j & 1) == 0) {
            if (QK) {
                const int op = j >> 1, mb = op >> 3, ks = op & 7;
                f32x16 &acc = fs.S[(2 * PAR + 1 + mb) & 3];
                if (ks == 0) mfma_first(acc, fr[j & 3], qf[ks]);
                else mfma_v(acc, fr[j & 3], qf[ks]);
            }
        } else {
            if (PV) {
                const int op = j >> 1, kk = op >> 2, db = op & 3;
                mfma_a(o[db], fr[j & 3], Pnxt[kk]);
            }
        }
        TC_SB();
    }
    step_fence_out(o, fs.S);
    // the stream's last stages (positions 27..31) run in the first slots of the next step
    l_cur = lc;
    l_nxt = ln;
#undef TC_OPADDR
#undef TC_OPLOAD
#undef TC_SREG
}

// Runs the pipelined path over tiles [0, n) of the item's range (all full prefix tiles) and leaves
// the row state as the general loop keeps it (reference in m_run).  Returns false (work-group
// uniform) when a weight overflowed: the caller then redoes the item from scratch in the general loop.
__device__ __forceinline__ bool fast_tiles(RowState<1> &st, const bf16x8 (&qf)[1][8], const Geom &g,
                                           const BatchDev &b, const AttnArgs &a, const AttnItem &it, char *lds,
                                           int32_t *s_bid, int n, int tid)
{
    const int lane = tid & 63, r32 = lane & 31, hh = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const float c = a.scale_log2;
    const char *pool_l = g.pool + (int64_t)a.layer * g.layer_stride + (int64_t)it.kvh * kHeadBlk;
    const int64_t bb = g.block_bytes;
    const uint32_t v_half = (uint32_t)(g.block_bytes >> 1);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;

    // ---- loads: wave w brings block w of a tile (16 keys): K as four 1 KB pieces of four rows each,
    // chunk c of row r stored at chunk position c ^ r; V verbatim (4 KB per block and head)
    // (the per-lane offsets are recomputed at every use rather than kept in registers across the steps)
    // Only tiles that exist are loaded, and the waits below count exactly the loads that may still
    // be in flight (s_waitcnt vmcnt tells which tiles have landed because a wave's loads complete in
    // issue order).
    auto issue_k = [&](int buf, int bid) {
        const char *src = pool_l + (int64_t)entry_bid(__builtin_amdgcn_readfirstlane(bid)) * bb;
        const uint32_t dst = lds0 + buf * kFastKTile + w * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rb = 4 * i + (lane >> 4);
            load_to_lds(dst + i * 1024, src, rb * 256 + (((lane & 15) ^ rb) * 16));
        }
    };
    auto issue_v = [&](int buf, int bid) {
        const char *src = pool_l + (int64_t)entry_bid(__builtin_amdgcn_readfirstlane(bid)) * bb + v_half;
        const uint32_t dst = lds0 + kFastV + buf * kVTile + w * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i) load_to_lds(dst + i * 1024, src + i * 1024, lane * 16);
    };
    // wait until at most k batches (one tile's K or V: 4 loads per wave) are still in flight
    auto wait_batches = [&](int k) {
        if (k <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (k == 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else if (k == 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else if (k == 3) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
        else if (k == 4) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(20)" ::: "memory");
    };
    // the item carries the block ids of its first four tiles
    auto item_bid = [&](int t) {
        const int b0 = it.bid[4 * t], b1 = it.bid[4 * t + 1], b2 = it.bid[4 * t + 2], b3 = it.bid[4 * t + 3];
        return w == 0 ? b0 : w == 1 ? b1 : w == 2 ? b2 : b3;
    };
    issue_k(0, item_bid(0));                            // n >= 3: tiles 0, 1, 2 exist
    issue_k(1, item_bid(1));
    issue_k(2, item_bid(2));
    issue_v(0, item_bid(0));
    if (3 < n) issue_k(3, item_bid(3));
    issue_v(1, item_bid(1));
    // the block-id table is filled behind these loads, so that its round trip to the block table
    // does not delay them (the barrier of the prime step publishes it)
    fill_bids(s_bid, b, it, tid);

    // ---- operand read addresses (LDS byte addresses, 32 bit)
    // chunk (2 ks + hh) ^ (r32 & 15) of row r32: the k-step only flips bits 5..7 of the byte address
    uint32_t kb = lds0 + r32 * 256 + ((hh ^ (r32 & 15)) << 4);
    uint32_t vb = lds0 + kFastV + r32 * 32 + hh * 16;

    FastState fs;
    fs.l = 0.f;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int e = 0; e < 4; ++e) { fs.pE[kk][e] = 0u; fs.pO[kk][e] = 0u; }

    // ---- prime: QK(0) from K buffer 0; reference; weights of keys 0..31
    wait_batches(4 + (3 < n ? 1 : 0));                  // everything issued after K(0) may still be in flight
    __syncthreads();                                    // K(0) landed for every wave; block ids visible
    {
        typedef const __attribute__((address_space(3))) bf16x8 *lds_frag;
        f32x16 z;
#pragma unroll
        for (int e = 0; e < 16; ++e) z[e] = 0.f;
        fs.S[3] = z;
        fs.S[0] = z;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            fs.S[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(lds_frag)(uintptr_t)(kb ^ (ks << 5)), qf[0][ks], fs.S[3], 0, 0, 0);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            fs.S[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(lds_frag)(uintptr_t)((kb ^ (ks << 5)) + 32 * 256), qf[0][ks], fs.S[0], 0, 0, 0);
        // reference: the largest score among the run's first 32 keys - its real ones: the unused tail
        // of an aliased table block holds zero keys, whose score 0 says nothing about the row
        const int pad0 = entry_pad(it.bid[0]), pad1 = entry_pad(it.bid[1]);
        float mx;
        if ((pad0 | pad1) == 0) {
            mx = fs.S[3][0];
#pragma unroll
            for (int e = 1; e < 16; ++e) mx = fmaxf(mx, fs.S[3][e]);
        } else {
            mx = -INFINITY;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int t = 8 * ((e >> 2) & 1) + 4 * hh + (e & 3);
                if (t < 16 - ((e >> 3) ? pad1 : pad0)) mx = fmaxf(mx, fs.S[3][e]);
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        st.m_run[0] = mx * c;
        fs.nm = -st.m_run[0];
        // weights of keys 0..31, left in the state the steps' stream expects at a step's start: the last
        // five scores are in flight (27: summed, not packed; 28: exponentiated; 29: scaled; 30, 31: raw)
#pragma unroll
        for (int e = 0; e < 14; ++e) fs.S[3][e] = fmaf(fs.S[3][e], c, fs.nm);
#pragma unroll
        for (int e = 0; e < 13; ++e) fs.S[3][e] = __builtin_amdgcn_exp2f(fs.S[3][e]);
#pragma unroll
        for (int e = 0; e < 12; ++e) fs.l += fs.S[3][e];
#pragma unroll
        for (int d = 0; d < 5; ++d) {
            uint32_t pk;
            v_pack(pk, fs.S[3][2 * d], fs.S[3][2 * d + 1]);
            fs.pE[d >> 2][d & 3] = pk;
        }
    }

    // ---- steps.  Before step s: K reads go to buffer (s+1) & 3, V reads to buffer (s-1) & 3.
    // boundary after step s (s = -1 for the prime step)
    // The next step reads K(s+2) and V(s).  Issue order: K0 K1 K2 V0 [K3] V1, then per boundary b
    // K(b+5), V(b+3) (those that exist); what was issued after the later of the two needed tiles may
    // stay in flight.
    auto boundary = [&](int s, int bid_k, int bid_v) {
        if (s >= 0 && s + 5 < n) {                       // the steady state: one test, everything exists
            asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
            __syncthreads();
            issue_k((s + 1) & 3, bid_k);
            issue_v((s + 3) & 3, bid_v);
            return;
        }
        const int younger = s < 0 ? 3 + (3 < n ? 1 : 0)
                                  : (s + 1 < n ? 1 : 0) + (s + 2 < n ? 1 : 0) + (s + 3 < n ? 1 : 0) + (s + 4 < n ? 1 : 0);
        wait_batches(younger);
        __syncthreads();
        if (s + 3 < n) {
            if (s + 5 < n) issue_k((s + 1) & 3, bid_k);
            issue_v((s + 3) & 3, bid_v);
        }
    };
    auto advance = [&](int s_next) {                    // read addresses for step s_next
        const int dk = ((s_next + 1) & 3) == 0 ? -3 * kFastKTile : kFastKTile;
        const int dv = ((s_next - 1) & 3) == 0 ? -3 * kVTile : kVTile;
        kb += dk;
        vb += dv;
    };
    // block ids for the loads of a boundary are fetched from LDS one step early
    auto bid_of = [&](int t) { return s_bid[min(t, n - 1) * 4 + w]; };
    {
        const int bk = bid_of(4), bv = bid_of(2);
        boundary(-1, bk, bv);
    }
    // step 0 reads K buffer 1 and (nothing from) V buffer 3
    kb += kFastKTile;
    vb += 3 * kVTile;
    // step s with the matrix work that exists for it; then its boundary
#define TC_STEP(PAR_, QK_, PV_, s_)                                                               \
    {                                                                                             \
        const int ss_ = (s_);                                                                     \
        const int bk = bid_of(ss_ + 5), bv = bid_of(ss_ + 3);                                     \
        float l_cur, l_nxt;                                                                       \
        fast_step<PAR_, QK_, PV_>(fs, st.o[0], qf[0], kb, vb, c, l_cur, l_nxt);                   \
        fs.l += (ss_ < n ? l_cur : 0.f) + (ss_ + 1 < n ? l_nxt : 0.f);                            \
        if (ss_ < n) {                                                                            \
            boundary(ss_, bk, bv);                                                                \
            advance(ss_ + 1);                                                                     \
        }                                                                                         \
    }
    TC_STEP(0, true, false, 0)                          // n >= 3: tile 1 exists
    int s = 1;
    for (; s + 1 <= n - 2; s += 2) {                    // steady state: steps 1 .. n-2
        TC_STEP(1, true, true, s)
        TC_STEP(0, true, true, s + 1)
    }
    if (s <= n - 2) {
        TC_STEP(1, true, true, s)
        TC_STEP(0, false, true, s + 1)                  // step n-1: no tile n
        TC_STEP(1, false, true, s + 2)                  // step n: PV of the last tile
    } else {
        TC_STEP(1, false, true, s)
        TC_STEP(0, false, true, s + 1)
    }
#undef TC_STEP
    // Unused tails of aliased table blocks inside the run: their keys and values are zeros, so they
    // added nothing to O and, each, exactly 2^(0 c - ref) to the row sum - taken out here instead of
    // masking scores in every step.  That is only sound while this weight is small against the sum:
    // with ref >= 0 it is at most 1, and the sum holds the reference key's own weight 1.  A row whose
    // reference is negative sends the item to the general loop, which masks.
    bool bad = false;
    if (it.n_pad_fast > 0) {
        if (hh == 0) fs.l -= (float)it.n_pad_fast * __builtin_amdgcn_exp2f(fs.nm);
        bad = fs.nm > 0.f;
    }
    st.l_lane[0] = fs.l;
    // a weight that overflowed shows in the sum (inf or nan)
    const float l_row = fs.l + __shfl_xor(fs.l, 32);
    return __syncthreads_or(bad || !(l_row < 1e30f)) == 0;
}

// The kernel for one row block per wave: pipelined path over the leading run of full prefix tiles,
// general loop for the rest (ragged last prefix tile, causal suffix tiles, short ranges).
__global__ __launch_bounds__(256, 1) void attn_bf16_pipe_kernel(Geom g, BatchDev b, AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    int32_t *s_bid = (int32_t *)(lds + kFastBid);

    if ((int)blockIdx.x >= a.n_items) {                // extra work-groups: append the suffix to the pool
        append_unit<true>(g, b, a.layer, (const char *)a.k_new, (const char *)a.v_new,
                          blockIdx.x - a.n_items, threadIdx.x);
        return;
    }
    const AttnItem it = a.items[blockIdx.x];
    if (it.q < 0) return;                              // padding item (uniform for the work-group)
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    ItemRows<1> ir;
    item_rows<1>(ir, g, it, w, lane & 31);
    bf16x8 qf[1][8];
    load_q<1>(qf, g, a, it, ir, lane >> 5);
    RowState<1> st;
    reset_rows<1>(st);
    // leading full prefix tiles of the range
    const int n_fast = min(it.tile_end, it.P >> 6) - it.tile_begin;
    // (the XOR addressing of the K buffers needs the dynamic LDS segment 256-byte aligned)
    if (n_fast >= kFastMinTiles && ((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds & 255u) == 0) {
        const bool ok = fast_tiles(st, qf, g, b, a, it, lds, s_bid, n_fast, tid);
        // Everything below is derived from a thread id the compiler cannot connect with the one
        // above, so that none of it (row geometry, the general loop's per-thread offsets) is
        // computed early and kept in registers across the pipelined path.
        int tid2 = tid;
        asm volatile("" : "+v"(tid2));
        item_rows<1>(ir, g, it, tid2 >> 6, tid2 & 31);
        if (ok) {
            if (it.tile_begin + n_fast < it.tile_end)
                tile_loop<1, true>(st, qf, g, b, a, it, ir, lds, s_bid, n_fast, false, tid2);
        } else {
            reset_rows<1>(st);
            tile_loop<1, true>(st, qf, g, b, a, it, ir, lds, s_bid, 0, false, tid2);
        }
        store_rows<1>(st, g, a, it, ir, tid2 >> 6, tid2 & 63);
    } else {
        tile_loop<1, true>(st, qf, g, b, a, it, ir, lds, s_bid, 0, true, tid);
        store_rows<1>(st, g, a, it, ir, w, lane);
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
    static PerDeviceOnce configured;
    const hipError_t e = configured.run([] {
        return hipFuncSetAttribute((const void *)attn_bf16_kernel<RB>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    });
    if (e != hipSuccess) return e;
    TC_LAUNCH(attn_bf16_kernel<RB>, a.n_items + a.n_append, kLdsBytes, L, g, b, a);
    return hipGetLastError();
}

hipError_t launch_attn_bf16(const Geom &g, const BatchDev &b, const AttnArgs &a, int row_blocks, bool pipelined,
                            const Launch &L)
{
    if (a.n_items + a.n_append == 0) return hipSuccess;
    if (g.D != 128 || g.esize != 2) return hipErrorInvalidValue;
    if (row_blocks == 1 && pipelined) {
        static PerDeviceOnce configured;
        const hipError_t e = configured.run([] {
            return hipFuncSetAttribute((const void *)attn_bf16_pipe_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kLdsBytesPipe);
        });
        if (e != hipSuccess) return e;
        TC_LAUNCH(attn_bf16_pipe_kernel, a.n_items + a.n_append, kLdsBytesPipe, L, g, b, a);
        return hipGetLastError();
    }
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
