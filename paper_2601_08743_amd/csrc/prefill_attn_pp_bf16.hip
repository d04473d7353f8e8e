// Suffix prefill attention (App. E.4: the suffix attends to all stitched table content and causally
// to itself), bf16, for launches of many work items: 256 rows per work-group, eight waves in two
// groups that alternate between matrix work and vector work.
//
// The general kernel runs QK^T, softmax and PV of a key tile one after the other in every wave, and
// its barriers keep the four waves of a work-group in step, so the matrix cores idle through every
// softmax (~1000 vector cycles per tile and wave against 1024 matrix cycles).  Here a SIMD holds two
// waves of the SAME work-group, one from each group, and every barrier flips their roles:
//
//   interval      0        1        2        3        4       ...
//   group A     M(0)     V(0)     M(1)     V(1)     M(2)
//   group B      -       M(0)     V(0)     M(1)     V(1)
//
// M(t): S^T = K(t) Q^T and O^T += V(t-1)^T P(t-1)^T - 32 matrix instructions with their operand
// reads; V(t): mask, running maximum, exponentials, row sums, weights packed to bf16.  While one
// wave of a SIMD feeds the matrix core the other one runs its softmax.
//
// All keys come from the pool: the suffix is appended by a launch of its own BEFORE this kernel
// (a few microseconds, which is why this kernel is for long launches), so a query is one paged
// sequence of P + S keys, tiles of 64, and row (token s, head) sees keys 0 .. P + s.  Tiles travel
// global -> LDS directly (global_load_lds_dwordx4), two tiles ahead: a ring of three K buffers
// (rows of 256 B, 16-byte chunks XOR-swizzled by row as in the other kernels) and four V buffers;
// each wave brings 1/8 of a tile and waits for its own part before the barrier that publishes it.
//
// Rows: work-group rows m0 .. m0+255 of the (query, KV head) row space (row = token * G + head in
// group); wave w owns rows m0 + 32 w ...  Partials of split queries use the layout of the other
// bf16 kernels with eight 32-row blocks per group, which the merge kernel takes as a parameter.
#include "lds_dma.h"
#include "tc_internal.h"

namespace tc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

constexpr int kPpTile = kAttnKeys * 256;             // 16 KB: a K tile (64 rows of 256 B) or a V tile (4 x 4 KB)
constexpr int kPpKBufs = 3, kPpVBufs = 4;
constexpr int kPpV = kPpKBufs * kPpTile;             // V ring behind the K ring
constexpr int kPpBid = kPpV + kPpVBufs * kPpTile;    // block-table entries of the item's key range
constexpr int kPpLds = kPpBid + kPpMaxTiles * 4 * 4 + 256;   // + slack to align the rings to 256 B
constexpr int kPpRing = 5;                           // operand fragments in flight: reads run kPpRing - 1 matrix instructions ahead
constexpr float kPpRescale = 8.f;                    // log2 units: rescale O only when the maximum grew by more

// lanes l and l ^ 32 hold the two halves of one row: the larger of their two values, in both
// (v_permlane32_swap exchanges the upper 32 lanes of its first operand with the lower 32 of its
// second: with the same value in both it yields (low half twice, high half twice); no LDS round trip)
__device__ __forceinline__ float max_with_other_half(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// kPads: the batch has sequences that alias table slots, whose block-table entries carry unused
// tail positions to mask; without them a tile's entries are not looked at in the softmax phase.
template <bool kPads>
__global__ __launch_bounds__(512, 1) void attn_bf16_pp_kernel(Geom g, BatchDev b, AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    const AttnItem it = a.items[blockIdx.x];
    if (it.q < 0) return;                              // padding item (uniform for the work-group)
    // the XOR addressing of the K tiles needs them 256-byte aligned
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds_raw;
    const uint32_t pad = (256u - (lds_base & 255u)) & 255u;
    const uint32_t lds0 = lds_base + pad;
    int32_t *s_bid = (int32_t *)(lds_raw + pad + kPpBid);

    const int tid = threadIdx.x, lane = tid & 63, r32 = lane & 31, hh = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = w >> 2;                            // 0: group A, 1: group B (one interval behind)
    const int G = g.G, P = it.P, S = it.S;

    // ---- this lane's row
    const int m_rows = S * G;
    const int row_m = it.m0 + w * 32 + r32;
    const bool valid = row_m < m_rows;
    const int rm = valid ? row_m : m_rows - 1;
    const int s_tok = rm / G;
    const int head = it.kvh * G + (rm - s_tok * G);
    const int limit = P + s_tok;                       // last key this row sees
    // the wave's first row sees the fewest keys: tiles wholly below its limit need no mask
    const int wave_lim_min = P + min(it.m0 + w * 32, m_rows - 1) / G;
    // tiles of the range that any row of the work-group sees
    const int wg_lim_max = P + min(it.m0 + 255, m_rows - 1) / G;
    const int n = max(min(it.tile_end, (wg_lim_max >> 6) + 1) - it.tile_begin, 0);

    // ---- Q^T fragments (B operand): lane (row r32, half hh) holds q[row][16 ks + 8 hh .. +8]
    bf16x8 qf[8];
    {
        const char *qp = (const char *)a.q + ((int64_t)(it.cu + s_tok) * g.Hq + head) * 256 + hh * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = *(const bf16x8 *)(qp + ks * 32);
    }
    // ---- block-table entries of the range -> LDS (past the sequence: its last block, masked)
    {
        const int last_blk = max(((P + S + kBlockTokens - 1) >> 4) - 1, 0);
        const int32_t *bt = b.block_table + (int64_t)it.q * b.max_blocks;
        // (whole tiles below the sequence's last block go four entries per access where the table row
        // is 16-byte aligned; the rest entry by entry, clamped)
        const int32_t *src = bt + it.tile_begin * 4;
        const int n_wide = (((uintptr_t)src) & 15) == 0 ? max(min(n, (last_blk + 1 - it.tile_begin * 4) >> 2), 0) : 0;
        for (int idx = tid; idx < n_wide; idx += 512) ((int4 *)s_bid)[idx] = ((const int4 *)src)[idx];
        for (int idx = n_wide * 4 + tid; idx < n * 4; idx += 512) s_bid[idx] = bt[min(it.tile_begin * 4 + idx, last_blk)];
    }
    __syncthreads();

    // ---- loads: wave w brings two of the four 1 KB pieces of block (w / 2) of a tile, K and V
    const char *pool_l = g.pool + (int64_t)a.layer * g.layer_stride + (int64_t)it.kvh * 4096;
    const int64_t bb = g.block_bytes;
    const uint32_t v_half = (uint32_t)(g.block_bytes >> 1);
    // (the block id of the tile after the one being requested is read from LDS right behind the
    // loads and used by the next call, so that no call waits for an LDS round trip)
    int bid_next = s_bid[w >> 1];                      // tile 0 (never used when the range is empty)
    auto issue_tile = [&](int t) {                     // 4 load instructions; t = 0, 1, 2, .. in order
        const int j = w >> 1, i0 = 2 * (w & 1);
        const char *src = pool_l + (int64_t)entry_bid(__builtin_amdgcn_readfirstlane(bid_next)) * bb;
        const uint32_t kd = lds0 + (t % kPpKBufs) * kPpTile + j * 4096;
        const uint32_t vd = lds0 + kPpV + (t % kPpVBufs) * kPpTile + j * 4096;
#pragma unroll
        for (int i = i0; i < i0 + 2; ++i) {
            const int rb = 4 * i + (lane >> 4);       // row of the block; chunk c of row r goes to position c ^ r
            load_to_lds(kd + i * 1024, src, rb * 256 + (((lane & 15) ^ rb) * 16));
        }
#pragma unroll
        for (int i = i0; i < i0 + 2; ++i)               // V chunks in operand order (see v_off)
            load_to_lds(vd + i * 1024, src + v_half + i * 1024, (2 * (lane & 31) + (lane >> 5)) * 16);
        bid_next = s_bid[min(t + 1, n - 1) * 4 + j];
    };
    if (0 < n) issue_tile(0);
    if (1 < n) issue_tile(1);

    // ---- state
    f32x16 o[4], sacc[2];         // sacc: scores of the tile between its M and V phase
    bf16x8 pf[4];                 // weights of the tile between its V phase and the next M phase (always written first)
    bf16x8 vpre[kPpRing - 1];     // first V fragments of that M phase
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] = 0.f;
    float m_run = -INFINITY, l_lane = 0.f;
    const float c = a.scale_log2;
    typedef const __attribute__((address_space(3))) bf16x8 *lds_frag;
    const uint32_t k_off = r32 * 256 + ((hh ^ (r32 & 15)) << 4);
    // V: within each 1 KB (32 d-rows of 32 bytes) the loads fetch token half 0 of all rows, then half 1,
    // so that lane (row r32, half hh) reads position r32 + 32 hh = its lane number: 16 consecutive lanes
    // read 256 consecutive bytes (at the rows' own 32-byte pitch they would hit half the banks twice)
    const uint32_t v_off = kPpV + lane * 16;

    // M(t): PV(t-1) first - it uses up the weights, whose registers the new scores can then take -
    // then QK(t); operand fragments are read kPpRing - 1 matrix instructions ahead (an LDS round trip
    // is longer than two of them)
    auto m_phase = [&](int t, bool do_qk, bool do_pv) {
        const uint32_t kb = lds0 + (t % kPpKBufs) * kPpTile + k_off;
        const uint32_t vb = lds0 + ((t + kPpVBufs - 1) % kPpVBufs) * kPpTile + v_off;
        // the wave in its matrix phase goes first when both waves of a SIMD have an instruction to
        // issue (measured on one machine against the same build without it: -1.1 %)
        __builtin_amdgcn_s_setprio(2);
        bf16x8 kf[kPpRing];
#define TC_KF(j) (*(lds_frag)(uintptr_t)((kb ^ (((j) >> 1) << 5)) + ((j) & 1) * 32 * 256))
        if (do_pv) {
            bf16x8 vf[kPpRing];
#define TC_VF(j) (*(lds_frag)(uintptr_t)(vb + ((j) >> 2) * 4096 + ((j) & 3) * 1024))
#pragma unroll
            for (int j = 0; j < kPpRing - 1; ++j) vf[j] = vpre[j];      // read at the end of the softmax phase before
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (j + kPpRing - 1 < 16) vf[(j + kPpRing - 1) % kPpRing] = TC_VF(j + kPpRing - 1);
                else if (do_qk) kf[j + kPpRing - 1 - 16] = TC_KF(j + kPpRing - 1 - 16);   // the first K fragments ride behind the last V ones
                o[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[j % kPpRing], pf[j >> 2], o[j & 3], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);     // keep the reads where they are: ahead (the scheduler pulls them back to their use)
            }
#undef TC_VF
        }
        if (do_qk) {
            f32x16 zero;                               // the first product of each half starts from the constant 0
#pragma unroll
            for (int e = 0; e < 16; ++e) zero[e] = 0.f;
            if (!do_pv) {
#pragma unroll
                for (int j = 0; j < kPpRing - 1; ++j) kf[j] = TC_KF(j);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (j + kPpRing - 1 < 16) kf[(j + kPpRing - 1) % kPpRing] = TC_KF(j + kPpRing - 1);
                sacc[j & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j % kPpRing], qf[j >> 1], j < 2 ? zero : sacc[j & 1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __builtin_amdgcn_s_setprio(0);
#undef TC_KF
    };
    // V(t): scores of tile t -> weights.  (With unused block tails to mask, the tile's four
    // block-table entries are read from LDS at the end of the phase before, like the first V fragments.)
    int4 e4_next = make_int4(0, 0, 0, 0);
    if (kPads && n > 0) e4_next = *(const int4 *)&s_bid[0];
    auto v_phase = [&](int t) {
        const int key0 = (it.tile_begin + t) * kAttnKeys;
        int pad4 = 0;
        if (kPads) {
            const int4 e4 = e4_next;
            pad4 = entry_pad(e4.x) | (entry_pad(e4.y) << 8) | (entry_pad(e4.z) << 16) | (entry_pad(e4.w) << 24);
        }
        if (pad4 != 0 || key0 + kAttnKeys - 1 > wave_lim_min) {      // causal edge or unused block tails in this tile
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int in_blk = 8 * ((e >> 2) & 1) + 4 * hh + (e & 3);
                    const int pd = (pad4 >> (8 * (2 * mb + (e >> 3)))) & 255;
                    const int key = key0 + 32 * mb + 8 * (e >> 2) + 4 * hh + (e & 3);
                    const bool dead = (key > limit) | (in_blk >= kBlockTokens - pd);
                    sacc[mb][e] = dead ? -INFINITY : sacc[mb][e];
                }
        }
        float mx = sacc[0][0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sacc[0][e]);
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[1][e]);
        mx = max_with_other_half(mx);
        const float mxs = mx * c;
        if (__builtin_expect(__any(mxs > m_run + kPpRescale), 0)) {   // rare; also taken while m_run is still -inf
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
                sacc[mb][e] = __builtin_amdgcn_exp2f(fmaf(sacc[mb][e], c, neg_m));
            }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[kk][e] = (__bf16)sacc[kk >> 1][8 * (kk & 1) + e];
        // the row sum is taken over the weights as PV will use them (rounded to bf16), two per
        // instruction: v_dot2_f32_bf16 with (1, 1) as the other operand
        {
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            bf16x2 ones;
            ones[0] = (__bf16)1.f;
            ones[1] = (__bf16)1.f;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    bf16x2 pr;
                    pr[0] = pf[kk][e];
                    pr[1] = pf[kk][e + 1];
                    l_lane = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, l_lane, false);
                }
        }
        // the next matrix phase starts with PV of this tile: its first V fragments (as many as its
        // reads run ahead) are fetched now, so that it starts without waiting for an LDS round trip
        const uint32_t vb = lds0 + (t % kPpVBufs) * kPpTile + v_off;
#pragma unroll
        for (int j = 0; j < kPpRing - 1; ++j) vpre[j] = *(lds_frag)(uintptr_t)(vb + j * 1024);
        if (kPads) e4_next = *(const int4 *)&s_bid[min(t + 1, n - 1) * 4];
    };
    // the wave's own part of tile t must have landed before the barrier that lets the first wave
    // read it; the tile issued after it may still be in flight
    auto wait_tile = [&](int t) {
        if (t + 1 < n) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    };

    // ---- intervals (barrier to barrier).  Group A does M(t) in interval 2t and V(t) in 2t+1, group B
    // one interval later: both run the same loop, B behind one extra barrier at the start and A
    // through one at the end.  Tile t is first read in interval 2t (A's M(t)): A's waves make sure of
    // their part at the end of their V(t-1), B's at the end of their M(t-1).  Tile t+2 is requested at
    // the start of a wave's V(t) (A: interval 2t+1, B: 2t+2); the buffers it goes to were last read in
    // interval 2t-1.
    // A wave none of whose 32 rows exists (the row space of a (query, KV head) rarely fills its last
    // 256-row tile) brings its share of every tile and passes every barrier, but runs neither matrix
    // nor softmax phase: on a chip whose clock is set by its power budget, work not done is time
    // gained by the others.  (Kept apart from the loop below, which compiles to worse code with a
    // test around its phases.)
    if (__builtin_amdgcn_readfirstlane((int)(it.m0 + w * 32 >= m_rows))) {
        if (n > 0) {
            wait_tile(0);
            __syncthreads();
            if (grp) __syncthreads();
            if (grp) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (2 < n) issue_tile(2);
            if (!grp) wait_tile(1);
            __syncthreads();
            for (int t = 1; t < n; ++t) {
                if (grp) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
                if (t + 2 < n) issue_tile(t + 2);
                if (!grp) wait_tile(t + 1);
                __syncthreads();
            }
            __syncthreads();
            if (!grp) __syncthreads();
        }
        return;
    }
    if (n > 0) {
        wait_tile(0);
        __syncthreads();                               // tile 0 visible
        if (grp) __syncthreads();
        m_phase(0, true, false);
        if (grp) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // tile 1 (B has requested nothing younger)
        __syncthreads();
        if (2 < n) issue_tile(2);
        v_phase(0);
        if (!grp) wait_tile(1);
        __syncthreads();
        for (int t = 1; t < n; ++t) {
            m_phase(t, true, true);
            if (grp) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // tile t+1
            __syncthreads();
            if (t + 2 < n) issue_tile(t + 2);          // in the softmax phase, which has the time to spare
            v_phase(t);
            if (!grp) wait_tile(t + 1);
            __syncthreads();
        }
        m_phase(n, false, true);                       // PV of the last tile
        __syncthreads();
        if (!grp) __syncthreads();
    }

    // ---- final normalisation and store: the output rows, or (split queries) this partition's partial
    const float l = l_lane + __shfl_xor(l_lane, 32);
    if (it.n_splits > 1) {
        const int64_t slot = (int64_t)it.split * it.n_groups + it.group;
        const float inv = l > 0.f ? 1.f / l : 0.f;
        f16x4 *po = (f16x4 *)a.part_o + ((slot * 8 + w) * 16) * 64 + lane;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                f16x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (_Float16)(o[db][4 * q4 + e] * inv);
                __builtin_nontemporal_store(v, &po[(db * 4 + q4) * 64]);
            }
        if (hh == 0) {
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            f32x2 ml;
            ml[0] = m_run;
            ml[1] = l;
            __builtin_nontemporal_store(ml, &((f32x2 *)a.part_ml)[(slot * 8 + w) * 32 + r32]);
        }
        return;
    }
    if (!valid) return;
    const int64_t row = (int64_t)(it.cu + s_tok) * g.Hq + head;
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
}

hipError_t launch_attn_pp_bf16(const Geom &g, const BatchDev &b, const AttnArgs &a, const Launch &L)
{
    if (a.n_items == 0) return hipSuccess;
    if (g.D != 128 || g.esize != 2 || a.n_append != 0) return hipErrorInvalidValue;
    static PerDeviceOnce configured;
    const hipError_t ec = configured.run([] {
        hipError_t e = hipFuncSetAttribute((const void *)attn_bf16_pp_kernel<false>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kPpLds);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)attn_bf16_pp_kernel<true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kPpLds);
        return e;
    });
    if (ec != hipSuccess) return ec;
    if (a.has_pads)
        hipExtLaunchKernelGGL(attn_bf16_pp_kernel<true>, dim3(a.n_items), dim3(512), kPpLds, L.stream, L.start, L.stop, 0, g, b, a);
    else
        hipExtLaunchKernelGGL(attn_bf16_pp_kernel<false>, dim3(a.n_items), dim3(512), kPpLds, L.stream, L.start, L.stop, 0, g, b, a);
    return hipGetLastError();
}

}  // namespace tc
