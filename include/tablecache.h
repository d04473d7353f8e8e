/*
 * libtablecache - the online hot path of TableCache on one MI355X (gfx950).
 *
 * The paper precomputes one KV cache per database table offline and keeps them
 * in CPU memory (Sec. 1, Sec. 4.1).  Online, per prompt, the KV caches of the
 * matched tables are brought to the GPU if they are not there (Sec. 4.2, App. A),
 * concatenated in match order (Sec. 4.1.2) and the model then computes only the
 * uncached rest of the prompt - question and instructions - which attends to all
 * of the table content before it (App. E.4).  This library is that path:
 *
 *   tc_register_table_kv   a table's precomputed KV in pinned host memory      (Sec. 1, 4.1)
 *   tc_load_async          make tables device-resident under a replacement rule (Sec. 4.2, 4.2.2, App. A)
 *   tc_stitch_kv           concatenate the selected tables' KV into paged blocks (Sec. 4.1.2)
 *   tc_prefill_attn        GQA attention of the suffix over stitched KV + itself (App. E.4)
 *
 * Conventions
 *   - Plain C ABI.  Every pointer argument says HOST or DEVICE.  No call throws or
 *     aborts; every call returns a tc_status (0 = ok, negative = error) and, on an
 *     argument or state error, has no side effect (a failed tc_stitch_kv allocates
 *     nothing).  tc_last_error() gives a text for the most recent failure.
 *   - Streams are hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued and the call returns; errors of asynchronous work surface as
 *     TC_ERR_HIP from a later call.
 *   - One host thread per context at a time, and one compute stream: tc_stitch_kv uploads the
 *     batch's integer plan on its stream, and the tc_prefill_attn calls of that batch must be
 *     ordered after it (same stream, or the caller's own event).
 *   - Element type: TC_F32 (fp32 storage and arithmetic) or TC_BF16 (bf16 storage,
 *     fp32 accumulation on the matrix cores).  bf16 needs head_dim == 128.
 *
 * The device KV pool
 *   The caller allocates one device buffer of tc_pool_bytes(cfg) bytes and hands it
 *   to tc_create.  It counts n_pool_blocks blocks of block_size (16) tokens in all layers.
 *   The first table_capacity * slot_blocks of them (slot_blocks = ceil(max_table_tokens /
 *   block_size)) form the TABLE region: slot s is one contiguous piece of slot_blocks *
 *   n_layers * tc_block_bytes(cfg) bytes holding one resident table as registered - its K
 *   rows [L][n_tokens][Hkv][D], then, at half the slot, its V rows - so a table (or a run
 *   of its layers) arrives as two large host->device transfers.  The remaining blocks are
 *   SEQUENCE blocks handed out by tc_stitch_kv, lowest-numbered free block first, stored
 *   layer-major behind the table region; their in-block layout is private to the library
 *   (read them back with tc_read_seq_kv).
 */
#ifndef TABLECACHE_H
#define TABLECACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tc_ctx tc_ctx;
typedef int32_t tc_status;

enum {
    TC_OK = 0,
    TC_ERR_INVALID = -1,       /* bad argument (null, out of range, unsupported shape)        */
    TC_ERR_UNKNOWN_TABLE = -2, /* table id was never registered                               */
    TC_ERR_OOM_POOL = -3,      /* not enough free sequence blocks (or max_blocks too small)   */
    TC_ERR_NOT_RESIDENT = -4,  /* a table needed by the call is not on the device             */
    TC_ERR_CAPACITY = -5,      /* table does not fit a slot / nothing can be evicted          */
    TC_ERR_HIP = -6            /* the HIP runtime reported an error                           */
};

enum { TC_F32 = 0, TC_BF16 = 1 };
enum { TC_POLICY_LRU = 0, TC_POLICY_FIFO = 1, TC_POLICY_LFU = 2 };
/* How the device cache keeps a table: as registered (token rows; sequences are built by copying,
 * tc_stitch_kv), or already in the pool's block layout, every table starting on a block of its own
 * (sequences are built by pointing at those blocks, tc_stitch_alias; bf16 only). */
enum { TC_SLOTS_ROWS = 0, TC_SLOTS_BLOCKS = 1 };

typedef struct {
    int32_t n_layers;          /* L                                                          */
    int32_t n_q_heads;         /* Hq, a multiple of n_kv_heads                               */
    int32_t n_kv_heads;        /* Hkv                                                        */
    int32_t head_dim;          /* D: 64 or 128 (bf16: 128)                                   */
    int32_t block_size;        /* tokens per block; must be 16                               */
    int32_t dtype;             /* TC_F32 | TC_BF16                                           */
    int64_t n_pool_blocks;     /* total blocks, table slots included                         */
    int32_t table_capacity;    /* C of App. A: how many tables the device cache holds        */
    int32_t max_table_tokens;  /* longest table that may be registered (sizes a slot)        */
    int32_t policy;            /* TC_POLICY_*                                                */
    int32_t slot_layout;       /* TC_SLOTS_*                                                 */
} tc_config;

/* Bytes of one block in one layer: 2 (K and V) * Hkv * block_size * D * sizeof(element). */
size_t tc_block_bytes(const tc_config *cfg);
/* Bytes the caller must allocate for the pool: n_layers * n_pool_blocks * tc_block_bytes, plus, with
 * TC_SLOTS_BLOCKS, room for one table as registered (host copies land there before they are laid out
 * into blocks).  0 if cfg is invalid. */
size_t tc_pool_bytes(const tc_config *cfg);
/* First sequence block = table_capacity * ceil(max_table_tokens / block_size).  -1 if cfg is invalid. */
int64_t tc_first_seq_block(const tc_config *cfg);

/*
 * Create a context over a caller-owned pool.
 *   cfg          HOST, copied.
 *   kv_pool_dev  DEVICE, 256-byte aligned, at least tc_pool_bytes(cfg) bytes, owned by the
 *                caller, must outlive the context.  Contents need not be initialised.
 *   out          HOST, receives the context.
 * The library allocates only small metadata buffers of its own (work lists, split-KV partials).
 */
tc_status tc_create(const tc_config *cfg, void *kv_pool_dev, size_t pool_bytes, tc_ctx **out);
tc_status tc_destroy(tc_ctx *ctx);

/*
 * Register a table's precomputed KV (Sec. 1: table KV computed offline and stored in CPU
 * memory; Sec. 4.1.2: a trie leaf names the table id and where its KV is kept).
 *   table_id  >= 0, unique.
 *   n_tokens  1 .. max_table_tokens.
 *   host_k, host_v  HOST, pinned (hipHostMalloc or torch pin_memory), layout
 *             [L][n_tokens][Hkv][D] in the context's element type, owned by the caller,
 *             must stay valid and unchanged until the context is destroyed.
 * Nothing is copied here.
 */
tc_status tc_register_table_kv(tc_ctx *ctx, int32_t table_id, int32_t n_tokens,
                               const void *host_k, const void *host_v);

/*
 * Request tables, in order, from the device table cache (Sec. 4.2: an update happens
 * only when a request targets a non-cached table and then swaps it in, the victim
 * chosen by the replacement rule; App. A gives the rules; Sec. 4.2.2: the copies run
 * concurrently with computation).  For each id, the rule's Update(request) is applied
 * exactly as listed in App. A; on a miss the table takes the lowest free slot, or the
 * victim's slot, and host->device copies of its K and V for layers [l0, l1) are
 * enqueued on `stream`.  A later call with another layer range for a table that is
 * already in the cache (a hit) copies the layers not copied yet.
 *   table_ids  HOST, n entries.
 *   stream     the side stream the copies run on.
 * Ordering against other streams is the library's job: a stitch that reads a slot
 * waits for that slot's copies; a copy into a reused slot waits for the last stitch
 * that read it.  The (table, hit, evicted) trace is kept for tc_load_trace.
 * A pinned table (tc_pin_tables) is never the victim: the rule's first choice among
 * the unpinned tables goes instead; TC_ERR_CAPACITY if a miss finds every cached table
 * pinned (ids before it in the list stay requested).
 * Errors: TC_ERR_UNKNOWN_TABLE, TC_ERR_INVALID (layer range), TC_ERR_CAPACITY, TC_ERR_HIP.
 */
tc_status tc_load_async(tc_ctx *ctx, const int32_t *table_ids, int32_t n,
                        int32_t l0, int32_t l1, void *stream);

/*
 * Pin / unpin tables in the device cache (reference counted, by table id; a table need
 * not be cached yet).  App. A states each rule for one request at a time; the tables of
 * one query, and of a micro-batch whose copies were issued ahead of its computation
 * (Sec. 4.2.2), must all still be cached when the stitch runs, which the literal rules
 * do not guarantee (FIFO can drop a table that was a hit a moment ago, LFU drops the
 * table it has just inserted).  A caller pins a request's tables before requesting them
 * and unpins them once its stitch is enqueued.  With nothing pinned the rules are
 * exactly App. A's.   table_ids  HOST, n entries.
 * Errors: TC_ERR_UNKNOWN_TABLE; TC_ERR_INVALID (unpin of a table that is not pinned:
 * nothing is changed).
 */
tc_status tc_pin_tables(tc_ctx *ctx, const int32_t *table_ids, int32_t n);
tc_status tc_unpin_tables(tc_ctx *ctx, const int32_t *table_ids, int32_t n);

/* Copy out up to `cap` entries of the access trace since the last call: triples
 * (table, hit 0/1, evicted table or -1).  HOST out[3*cap].  Returns the count (>= 0). */
int32_t tc_load_trace(tc_ctx *ctx, int32_t *out, int32_t cap);
/* 1 if the table is in the device cache with layers [l0,l1) copied (or enqueued), else 0. */
int32_t tc_is_resident(const tc_ctx *ctx, int32_t table_id, int32_t l0, int32_t l1);

/*
 * Stitch (Sec. 4.1.2: the KV caches of the tables found in the prompt are concatenated,
 * in the order they were found, and fed to the model).  For query i the tables
 * table_ids[cu_tables[i] .. cu_tables[i+1]) give P_i = sum of their lengths schema
 * tokens; ceil((P_i + suffix_len[i]) / 16) sequence blocks are taken (lowest free
 * first, queries in order), and a gather kernel copies, for every layer and KV head,
 * logical token p of the concatenation into slot p % 16 of block block_table[i][p / 16].
 * Slots past P_i in the touched blocks are zero-filled.  A table may appear twice.
 *   table_ids, cu_tables, suffix_len   HOST in  (cu_tables has B+1 entries)
 *   block_table                        HOST out [B][max_blocks], unused entries -1
 *   prefix_len                         HOST out [B]
 *   stream                             the compute stream; the gather is enqueued on it
 * The batch becomes the context's current batch (its integer plan is uploaded once and
 * reused by tc_prefill_attn for every layer).
 * Errors: TC_ERR_UNKNOWN_TABLE, TC_ERR_NOT_RESIDENT (all layers must be resident or
 * enqueued), TC_ERR_OOM_POOL, TC_ERR_INVALID.
 */
tc_status tc_stitch_kv(tc_ctx *ctx, const int32_t *table_ids, const int32_t *cu_tables, int32_t B,
                       const int32_t *suffix_len, int32_t *block_table, int32_t max_blocks,
                       int32_t *prefix_len, void *stream);

/*
 * Stitch without copying (contexts created with TC_SLOTS_BLOCKS).  Sec. 1 criticises prefix caches
 * for keeping a copy of the shared schema per request; here the concatenation of Sec. 4.1.2 is made
 * in the block table alone: query i's sequence lists, table by table in match order, the blocks of
 * the slots that hold its tables, then ceil(S_i / 16) blocks of its own for the suffix.  No kernel
 * runs and no table byte moves.  A table of n tokens fills ceil(n / 16) blocks; the unused positions
 * at the end of its last block hold zero keys and values and take no part in attention (the library
 * remembers where they are), so the sequence is as long as its blocks:
 *   prefix_len[i] = 16 * (number of table blocks of query i)       (>= the sum of the table lengths)
 * and this padded length is what tc_prefill_attn must be given.  Arguments and errors as for
 * tc_stitch_kv; block_table entries below tc_first_seq_block are blocks of table slots (slot s owns
 * s * ceil(max_table_tokens / 16) onwards).  Whatever is enqueued on `stream` afterwards runs after
 * the loads of the tables it reads.  The tables must stay cached until the batch's last attention
 * launch has been enqueued (pin them, tc_pin_tables); a later load that evicts one of them waits on
 * its own stream for those launches.  tc_release_seqs gives back the suffix blocks only.
 * Keys are used as stored: this entry point does not re-encode positions.
 */
tc_status tc_stitch_alias(tc_ctx *ctx, const int32_t *table_ids, const int32_t *cu_tables, int32_t B,
                          const int32_t *suffix_len, int32_t *block_table, int32_t max_blocks,
                          int32_t *prefix_len, void *stream);

/*
 * Stitch with positional re-encoding (Sec. 4.1.1, last paragraph: table KV is stored without
 * positional encoding, and at inference every token is encoded by its global position in the
 * concatenated sequence).  Same as tc_stitch_kv, except that the registered keys are taken to be
 * position-free and each key row is written to the pool rotary-encoded for position
 * pos0[i] + p, p being the token's index in query i's concatenation: in every head, elements
 * (j, j + D/2) are turned by (pos0[i] + p) * rope_theta^(-2j/D) radians (the half-split convention
 * of the rotary-position decoders the paper evaluates).  Values are copied unchanged and so are
 * block tables and prefix lengths.  The turn is reduced in fp64, the rotation is fp32, the result
 * is rounded once to the element type.  The caller's q and k_new are expected to be encoded
 * already (for positions pos0[i] + P_i + s), as a model's attention layer produces them.
 *   pos0         HOST in [B], position of each query's first schema token; NULL = all zero
 *   rope_theta   the encoding's base (> 1), e.g. 1e6 or 1e4
 * Further errors: TC_ERR_INVALID for a bad base, a negative position or a head size whose
 * half is not a whole number of 16-byte chunks.
 */
tc_status tc_stitch_kv_rope(tc_ctx *ctx, const int32_t *table_ids, const int32_t *cu_tables, int32_t B,
                            const int32_t *suffix_len, const int32_t *pos0, double rope_theta,
                            int32_t *block_table, int32_t max_blocks, int32_t *prefix_len, void *stream);

/*
 * Suffix prefill attention, one layer (App. E.4: only the uncached part of the prompt
 * is computed, and it attends to all preceding table content; it is causal to itself).
 * First the suffix keys/values are appended to the sequence blocks at logical positions
 * [P_i, P_i + S_i); then for query i, head h (KV head h / (Hq/Hkv)), suffix row r:
 *   out = softmax_j( sm_scale * q . k_j ) v_j   over j in [0, P_i) U [P_i, P_i + r].
 *   q, out            DEVICE [sum S][Hq][D]      (16-byte aligned)
 *   k_new, v_new      DEVICE [sum S][Hkv][D]     (16-byte aligned)
 *   cu_seqlens        HOST [B+1], cu_seqlens[i+1]-cu_seqlens[i] == suffix_len[i]
 *   block_table       HOST [B][max_blocks]
 *   prefix_len, suffix_len   HOST [B]
 * The integer arguments normally are the ones tc_stitch_kv returned for the current
 * batch, in which case nothing is uploaded; if they differ, the call re-plans from them.
 * Every block id of such a batch must be a sequence block in range, or - with block-format slots
 * - a block of a slot that holds a fully loaded table, standing where the whole block lies below
 * prefix_len (a table block is only ever read); which positions of a table's last block hold
 * tokens follows from the table cached in that slot at the time of the call, so the tables of
 * sequences made by tc_stitch_alias must stay cached (pinned) for as long as those sequences are
 * attended to.
 * Errors: TC_ERR_INVALID, TC_ERR_HIP.
 */
tc_status tc_prefill_attn(tc_ctx *ctx, int32_t layer, const void *q, const void *k_new,
                          const void *v_new, void *out, const int32_t *cu_seqlens,
                          const int32_t *block_table, int32_t max_blocks,
                          const int32_t *prefix_len, const int32_t *suffix_len, int32_t B,
                          float sm_scale, void *stream);

/*
 * tc_prefill_attn for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results
 * as tc_prefill_attn; the difference is where the library keeps its own working memory for the call
 * - the batch's integer plan (work items, block tables, lengths) and the split-KV partials.
 * tc_prefill_attn puts them in buffers it allocates and grows on demand; this entry point puts them
 * in a fixed 64 MiB workspace that the library's code object carries (4 MiB plan, 60 MiB partials;
 * one copy per GPU, held until the process ends) and calls no hipMalloc, hipFree or other allocating
 * routine.  A batch whose plan or partials do not fit is refused with TC_ERR_CAPACITY and nothing
 * is enqueued (for scale: c2 needs 0.1 MiB + 7.6 MiB, a c5 micro-batch of 8 queries 0.5 + 21.6 MiB;
 * c3 and c4 run unsplit and need no partials).
 * Every call re-plans from its integer arguments unless they equal those of the previous call
 * through this entry point (a batch stitched by tc_stitch_kv is planned again here, once).
 * All contexts on one GPU share that GPU's workspace, which keeps the last call's contents (nothing
 * in it has to start at zero: every partial a merge reads was written by the attention launch
 * before it): calls through this entry point that overlap on one GPU - different streams, different
 * contexts - race; keep them on one stream or order them with events.
 * Errors: as tc_prefill_attn, plus TC_ERR_CAPACITY.
 */
tc_status tc_prefill_attn_noalloc(tc_ctx *ctx, int32_t layer, const void *q, const void *k_new,
                                  const void *v_new, void *out, const int32_t *cu_seqlens,
                                  const int32_t *block_table, int32_t max_blocks,
                                  const int32_t *prefix_len, const int32_t *suffix_len, int32_t B,
                                  float sm_scale, void *stream);

/*
 * Grow sequences for decoding: make sure query i's row of block_table has a block for every
 * position below new_len[i] (its current blocks are the leading entries that are not -1; more
 * are taken lowest-free-first, queries in order).  A decode step is then tc_prefill_attn with
 * suffix_len = 1 and prefix_len = everything already in the pool (the tables' tokens, the prompt's
 * own suffix, the tokens generated so far): the call appends the new token's K/V at position
 * prefix_len and attends to all of it.  Works for sequences made by tc_stitch_kv and by
 * tc_stitch_alias alike (for the latter prefix_len counts the padded positions, as returned by
 * the stitch; entries naming table blocks are left as they are).
 *   block_table  HOST in/out [B][max_blocks];  new_len  HOST in [B]
 * Errors: TC_ERR_OOM_POOL (max_blocks too small or no free block; nothing is changed),
 * TC_ERR_INVALID.
 */
tc_status tc_grow_seqs(tc_ctx *ctx, int32_t *block_table, int32_t max_blocks, int32_t B, const int32_t *new_len);

/* Return the sequence blocks named in block_table (HOST [B][max_blocks], -1 ignored) to
 * the free set.  The caller must have ordered this after the kernels that use them.
 * Errors: TC_ERR_INVALID if an entry is not an allocated sequence block (nothing freed). */
tc_status tc_release_seqs(tc_ctx *ctx, const int32_t *block_table, int32_t max_blocks, int32_t B);

/*
 * Read logical tokens [0, n_tokens) of one sequence in one layer back in token-major
 * order, undoing the private in-block layout: out_k, out_v HOST [n_tokens][Hkv][D].
 * blocks: HOST, ceil(n_tokens/16) sequence block ids.  Synchronises `stream`.
 * For checking the gather and the append bit for bit.
 */
tc_status tc_read_seq_kv(tc_ctx *ctx, int32_t layer, const int32_t *blocks, int32_t n_tokens,
                         void *out_k, void *out_v, void *stream);

/* Number of split-KV partitions tc_prefill_attn uses for the longest query of the
 * current batch (1 = no split); tc_set_kv_splits forces a value (0 = automatic). */
int32_t tc_kv_splits(const tc_ctx *ctx);
tc_status tc_set_kv_splits(tc_ctx *ctx, int32_t n_splits);
/* Rows per attention work-group of the bf16 kernel: 1 = 128 rows, 2 = 256 rows (each wave holds two
 * blocks of 32 rows and reuses every K/V fragment twice), 0 = automatic (256 when the batch still
 * yields enough work-groups to fill the chip).  Results do not depend on it beyond rounding. */
tc_status tc_set_row_blocks(tc_ctx *ctx, int32_t row_blocks);
/* Which bf16 attention kernel serves the batch: 0 = automatic (from the number and length of the
 * batch's work items), 1 = the general kernel (128 rows per work-group, register-staged K/V,
 * running-maximum softmax, two work-groups per CU), 2 = the pipelined kernel (128 rows,
 * direct-to-LDS K/V, fixed softmax reference with overflow fallback, one work-group per CU),
 * 3 = as 0 (the decode kernels serve batches in which no query brings more than one new token,
 * unless another kernel is forced: the keys of a KV head are split over waves and work-groups, a
 * second kernel combines them and adds the new token), 4 = the kernel for long launches (256
 * rows per work-group in two groups of waves that alternate between matrix and vector work; the
 * suffix is appended to the pool by a launch of its own before attention, which then reads all
 * keys from the pool; ignored while tc_set_row_blocks forces a row count).  Results do not depend
 * on it beyond rounding.  Invalidates the cached plan.
 * tc_attn_kernel reports the kernel of the current plan (1 .. 4; 0 when no plan is cached, for
 * fp32 contexts and for forced 256-row work-groups of the general kernel). */
tc_status tc_set_attn_kernel(tc_ctx *ctx, int32_t kind);
int32_t tc_attn_kernel(const tc_ctx *ctx);

/*
 * Measurement support.  With profiling on, every kernel the library launches carries two HIP
 * events that receive the begin and end timestamps of its own dispatch on the stream it is launched
 * on (no extra packets between kernels).  tc_profile_read waits for them and returns, per kernel kind (0 stitch, 1 append, 2 attention, 3 split-KV merge), the summed
 * elapsed milliseconds and the number of launches since the previous read.
 *   ms_out HOST double[4], count_out HOST int64_t[4].
 */
tc_status tc_profile_enable(tc_ctx *ctx, int32_t on);
tc_status tc_profile_read(tc_ctx *ctx, double *ms_out, int64_t *count_out);

/*
 * Front end (host only; upstream of the path): which tables does a prompt contain, and in which
 * order should a batch's queries run.
 *
 * Table Trie and Alg. 1 (Sec. 4.1.2): the token content of every table is inserted into a trie
 * whose terminal nodes hold the table id.  tc_trie_match scans a prompt's token sequence from
 * position 0: at position p it takes the longest table whose whole content is a prefix of the
 * rest of the prompt; if there is one, the table is reported and the scan continues behind it,
 * otherwise at p + 1.  The reported ids, in order, are the table_ids of tc_stitch_kv.
 *   tc_trie_insert   tokens HOST in [n_tokens] (n_tokens >= 1); TC_ERR_INVALID for a negative or
 *                    repeated id, an empty content, or a content equal to an inserted table's
 *   tc_trie_match    s HOST in [len]; table_ids_out / start_out HOST out [cap] (start_out may be
 *                    NULL): the matched tables and the positions where they start.  Returns the
 *                    number of matches (only the first cap are stored), or TC_ERR_INVALID.
 *
 * Query reranking (Sec. 4.2.1, Eq. 1-2): query i's tables as a bit set I_i over all n_tables
 * tables; d_ij = popcount(I_i xor I_j).  From the anchor (the paper draws it at random: the caller
 * passes it), the next query is always the remaining one nearest to the current one, lowest index
 * on ties.
 *   tc_rerank        table_ids / cu_tables HOST in, as for tc_stitch_kv (ids in [0, n_tables));
 *                    order_out HOST out [n_queries], the visiting order.
 */
typedef struct tc_trie tc_trie;
tc_trie *tc_trie_create(void);
void tc_trie_destroy(tc_trie *trie);
tc_status tc_trie_insert(tc_trie *trie, int32_t table_id, const int32_t *tokens, int32_t n_tokens);
int32_t tc_trie_match(const tc_trie *trie, const int32_t *s, int32_t len, int32_t *table_ids_out,
                      int32_t *start_out, int32_t cap);
tc_status tc_rerank(const int32_t *table_ids, const int32_t *cu_tables, int32_t n_queries, int32_t n_tables,
                    int32_t anchor, int32_t *order_out);

/*
 * Computation-loading pipeline schedule (Sec. 4.2.2): the ordered requests are computed
 * in micro-batches of b_c while the tables of up to the next b_m requests are copied in.
 * Host only.  The steps' compute ranges [compute_begin, compute_end) follow one another and
 * cover the batch; each holds b_c requests, fewer at the end of the batch (or with `taper`) or where the
 * distinct tables of b_c requests would not fit the cache together (the step is cut short
 * and the next one starts there).
 * Before a step's stitch the caller requests the tables of [demand_begin, demand_end) (those
 * of its requests that no earlier step prefetched: copies the computation has to wait
 * for); after its stitch is enqueued the caller unpins the step's tables and requests
 * those of [prefetch_begin, prefetch_end), which overlap the step's attention layers.
 * The prefetch range ends at compute_end + b_m, or earlier where the distinct tables of
 * the requests loaded but not yet computed would exceed `capacity` (they are pinned until
 * their stitch).  b_m = 0 gives the schedule without overlap.
 * keep_pinned != 0: the step's own tables stay pinned until its attention layers are enqueued
 * (tc_stitch_alias: the layers read the table slots in place), so they count against the cache
 * while the prefetch range is sized; the caller then unpins after the layers, not after the stitch.
 * taper != 0: towards the end of the batch a step takes min(b_c, max(1, remaining / 2)) requests
 * (.., b_c, b_c/2, .., 2, 1, 1).  When the copies are the bottleneck, what runs after the last
 * copy has landed is the computation of the final step; tapering makes that one request.
 *   table_ids, cu_tables   HOST, request i uses table_ids[cu_tables[i] .. cu_tables[i+1]).
 *   steps_out              HOST, room for `cap` steps; n_queries always suffice.
 * Returns the number of steps, or a negative tc_status: TC_ERR_INVALID (null pointers,
 * b_c < 1, b_m < 0, cap too small), TC_ERR_CAPACITY (a single request names more than
 * `capacity` distinct tables).
 */
typedef struct tc_pipe_step {
    int32_t compute_begin, compute_end;
    int32_t demand_begin, demand_end;
    int32_t prefetch_begin, prefetch_end;
} tc_pipe_step;
int32_t tc_plan_pipeline(const int32_t *table_ids, const int32_t *cu_tables, int32_t n_queries,
                         int32_t capacity, int32_t b_c, int32_t b_m, int32_t keep_pinned, int32_t taper,
                         tc_pipe_step *steps_out, int32_t cap);

/* Text for the most recent error on this context; library-owned, valid until the next call. */
const char *tc_last_error(const tc_ctx *ctx);
/* Library version string. */
const char *tc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TABLECACHE_H */
