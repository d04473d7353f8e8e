// Plain data shared by the host logic and the kernels of libtablecache: constants and the structures
// that travel to the device.  Nothing here needs the HIP headers, so the host-only parts (replacement
// rules, block allocator, attention planner) also build with a plain C++ compiler.
// Nothing here is part of the public ABI (see include/tablecache.h).
#pragma once
#include <stdint.h>

namespace tc {

constexpr int kBlockTokens = 16;     // tokens per pool block
constexpr int kAttnRows = 128;       // bf16 kernel: rows (suffix token x group head) per work-group and row block
constexpr int kAttnKeys = 64;        // bf16 kernel: keys per tile (4 pool blocks)
constexpr int kAttnMaxTiles = 256;   // bf16 kernel: key tiles per work item (block ids kept in LDS)
constexpr int kPpMaxTiles = 1024;    // the same for the long-launch kernel, which has the LDS to spare
constexpr int kPipeMaxTiles = 1024;  // and for the pipelined kernel (one work-group per CU)
constexpr int kF32Rows = 4;          // fp32 kernel: rows per work-group (one per wave)
constexpr int kF32Keys = 64;         // fp32 kernel: keys per tile

// Block-table entries as the kernels see them (device copies only; the caller's tables hold plain
// ids): the low 27 bits are the block id; the bits above count the unused token positions at the
// end of the block (0..15).  Only blocks of a table slot that a sequence aliases have any: a table
// of n tokens fills its last block up to n mod 16, the rest is zeros.
constexpr uint32_t kBidMask = (1u << 27) - 1;
constexpr int kPadShift = 27;
constexpr inline int32_t entry_bid(int32_t e) { return (int32_t)((uint32_t)e & kBidMask); }
constexpr inline int32_t entry_pad(int32_t e) { return (int32_t)((uint32_t)e >> kPadShift); }

// Pool geometry, passed by value to kernels.
struct Geom {
    char *pool;              // sequence region, biased so that block id b of layer l starts at
                             // pool + l * layer_stride + b * block_bytes (b counts from first_seq)
    int64_t layer_stride;    // bytes between the same sequence block in consecutive layers
    int64_t block_bytes;     // bytes of one block in one layer (K half then V half)
    char *tab_base;          // table region: slot s starts at tab_base + s * slot_bytes
    int64_t slot_bytes;      // bytes of one table slot, all layers (K part, then V part at half);
                             // layer l of a table of n tokens starts n * l * row_bytes into its part
    int32_t first_seq;       // first sequence block
    int32_t n_blocks;        // total blocks
    int32_t Hq, Hkv, D, G;
    int32_t esize;           // bytes per element
    int32_t row_bytes;       // Hkv * D * esize: one token's K (or V) row as registered
    int32_t head_bytes;      // D * esize
};

// One destination block of a stitch: 16 logical positions p0 .. p0+15 of query q.
struct StitchBlk {
    int32_t phys;      // destination block id
    int32_t seg;       // index (into the flattened segment arrays) of the segment holding p0
    int32_t p0;        // logical position of slot 0
    int32_t q;         // query index in the batch
};

// Device-side view of the current batch (all arrays int32, one upload per batch).
struct BatchDev {
    const int32_t *block_table;   // [B][max_blocks]
    const int32_t *cu_seqlens;    // [B+1]
    const int32_t *prefix_len;    // [B]
    const int32_t *suffix_len;    // [B]
    const int32_t *seg_start;     // [n_seg] logical start of segment within its query
    const int32_t *seg_len;       // [n_seg]
    const int32_t *seg_slot;      // [n_seg] table slot holding the segment's table
    const int32_t *seg_end_of_q;  // [B] one past the last segment index of query q
    const StitchBlk *stitch_blk;  // [n_stitch_blk]
    const int32_t *splits_of_q;   // [B] split-KV partitions used for query q
    const int32_t *tok_q;         // [sum S] query index of each suffix token
    const int32_t *rope_pos0;     // [B] position of each query's first schema token (re-encoding stitch), else null
    const double *rope_rev_freq;  // [D/2] theta^(-2i/D) / (2 pi): revolutions per position step, else null
    int32_t B, max_blocks, total_S, n_stitch_blk;
};

// One unit of attention work: a tile of rows of one (query, KV head) against a range of key tiles.
// Everything the work-group needs to start loading is in the item itself (one scalar fetch):
// the query's lengths and the block-table entries of its first four key tiles.
struct AttnItem {
    int32_t q;           // query index, -1 = padding item
    int32_t kvh;
    int32_t m0;          // first row (row = suffix_token * G + head_in_group)
    int32_t tile_begin;  // first key tile
    int32_t tile_end;    // one past the last key tile
    int32_t split;       // which partition this is (0 when n_splits == 1)
    int32_t n_splits;    // partitions of this query
    int32_t group;       // index of the (query, KV head, row tile): partial slots and arrival counter
    int32_t P, S, cu;    // prefix length, suffix length, first suffix row of the query
    int32_t n_groups;    // total number of groups in the batch
    int32_t bid[16];     // block-table entries of the first four key tiles of the range (clamped to the sequence)
    int32_t n_pad_fast;  // unused token positions inside the leading run of full prefix tiles of the range
    int32_t rsv[3];
};
static_assert(sizeof(AttnItem) == 128, "AttnItem layout");

// A (query, KV head, row tile) whose partitions the bf16 merge kernel combines.
struct MergeGroup {
    int32_t kvh, m0, n_splits, cu, S, pad[3];
};

struct AttnArgs {
    const void *q;
    const void *k_new;   // suffix keys / values [sum S][Hkv][D] of this layer
    const void *v_new;
    void *out;
    const AttnItem *items;
    float *part_o;       // split-KV partial outputs (layout and element type private to each kernel)
    float *part_ml;      // per partial row: (reference max in log2 units, sum of weights)
    float scale_log2;    // sm_scale * log2(e)
    int32_t layer;
    int32_t n_items;
    int32_t n_append;    // append units run by the bf16 attention launch (total_S + B), 0 = none
    int32_t has_pads;    // some block-table entry of the batch carries unused tail positions (aliased table blocks)
};

}  // namespace tc
