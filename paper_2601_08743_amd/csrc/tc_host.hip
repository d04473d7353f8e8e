// Host side of libtablecache: the C ABI of include/tablecache.h, the table registry, the
// device table cache with its replacement rules (paper App. A), the sequence-block allocator,
// per-batch planning (stitch descriptors, attention work list, split-KV) and kernel launches.
#include "../../include/tablecache.h"
#include "host_logic.h"
#include "tc_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <list>
#include <map>
#include <memory>
#include <mutex>
#include <set>
#include <string>
#include <unordered_map>
#include <vector>

using namespace tc;

namespace {

struct Table {
    int32_t n_tokens = 0;
    const char *host_k = nullptr, *host_v = nullptr;
    int32_t slot = -1;
    std::vector<uint8_t> layer_loaded;
};

struct Slot {
    int32_t table = -1;
    hipEvent_t ready = nullptr;        // recorded on the load stream after the latest copies
    hipStream_t ready_stream = nullptr;
    bool ready_pending = false;        // a record exists that other streams may have to wait for
    int32_t read_ev = -1;              // index into the read-event ring, -1 = never read
    uint32_t read_gen = 0;             // generation of that ring entry when the slot's stitch recorded it
    hipStream_t read_stream = nullptr; // stream of that stitch
    hipStream_t reader_stream = nullptr;   // block-format slots: stream of the last attention launch that
    bool reader_pending = false;           // read the slot through an aliasing sequence, not yet ordered
};

inline size_t align8(size_t n) { return (n + 7) & ~size_t(7); }

// ------------------------------------------------------------------ workspace of tc_prefill_attn_noalloc
// The entry point that allocates nothing keeps what tc_prefill_attn keeps in hipMalloc'ed buffers -
// the batch's integer plan and the split-KV partials - in this array, which the code object brings
// with it: 4 MiB for the plan, 60 MiB for partials.  Every GPU the library runs on holds its own
// copy at its own address until the process ends; host code reaches it only through the address
// hipGetSymbolAddress returns for the current device (tc_create resolves it once per device).
constexpr size_t kScratchPlanInts = size_t(1) << 20;
constexpr size_t kScratchPartFloats = size_t(15) << 20;
constexpr size_t kScratchBytes = (kScratchPlanInts + kScratchPartFloats) * 4;
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char *g_scratch_ptr[kMaxDevices];                   // device address of `scratch` on each device, once resolved

}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

struct tc_ctx {
    tc_config cfg{};
    Geom geom{};
    int32_t slot_blocks = 0;
    int64_t first_seq = 0;
    std::unordered_map<int32_t, Table> tables;
    std::unique_ptr<Replacement> rule;
    PinMap pins;                           // table -> pin count (> 0)
    std::vector<Slot> slots;
    std::set<int32_t> free_slots;
    SeqBlocks seq;                         // sequence blocks [first_seq, n_pool_blocks)
    std::vector<int32_t> trace;            // (table, hit, evicted) triples
    std::vector<hipEvent_t> read_ring;     // events recorded after stitch kernels
    std::vector<uint32_t> read_gen;        // how often each ring entry has been recorded
    int32_t read_next = 0;
    hipEvent_t raw_ev = nullptr;           // block-format slots: the raw staging area was last used up to here,
    hipStream_t raw_stream = nullptr;      // on this stream
    bool raw_pending = false;
    Plan plan;
    int32_t *h_stage = nullptr; size_t h_stage_ints = 0;
    int32_t *d_plan = nullptr; size_t d_plan_ints = 0;
    hipEvent_t stage_ev = nullptr; bool stage_pending = false;
    float *d_part = nullptr; size_t d_part_floats = 0;
    int device = 0;                        // the device the context was created on
    char *scratch_dev = nullptr;           // that device's copy of the static workspace (tc_prefill_attn_noalloc)
    char *d_read = nullptr; size_t d_read_bytes = 0;   // tc_read_seq_kv's staging, grown on demand
    PlanKnobs knobs;                       // tc_set_kv_splits / tc_set_row_blocks / tc_set_attn_kernel
    // per-kernel timing (tc_profile_*): pairs of events around launches, drained on read
    bool profiling = false;
    struct Timed { int kind; hipEvent_t a, b; };
    std::vector<Timed> timed;
    std::vector<hipEvent_t> ev_pool;
    double prof_ms[4] = {0, 0, 0, 0};
    int64_t prof_n[4] = {0, 0, 0, 0};
    std::string err;
};

namespace {

tc_status fail(tc_ctx *ctx, tc_status code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf;
    return code;
}

#define TC_HIP(ctx, call)                                                                       \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess)                                                                   \
            return fail(ctx, TC_ERR_HIP, "%s: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

hipEvent_t take_event(tc_ctx *ctx)
{
    hipEvent_t e = nullptr;
    if (!ctx->ev_pool.empty()) { e = ctx->ev_pool.back(); ctx->ev_pool.pop_back(); return e; }
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Record the next event of the read ring on `stream`; returns its index (-1 on error).
int32_t record_read(tc_ctx *ctx, hipStream_t stream)
{
    const int32_t ev = ctx->read_next;
    if (hipEventRecord(ctx->read_ring[ev], stream) != hipSuccess) return -1;
    ctx->read_next = (ctx->read_next + 1) % (int32_t)ctx->read_ring.size();
    ++ctx->read_gen[ev];
    return ev;
}

// Make `stream` wait for the last stitch that read slot `s`.  The ring entry the slot remembers may
// have been recorded again since (64 stitches later, possibly on another stream): then it no longer
// stands for that stitch, and a fresh event on the stitch's own stream - which covers everything
// enqueued there so far - takes its place.
hipError_t wait_for_reader(tc_ctx *ctx, Slot &s, hipStream_t stream)
{
    if (s.read_ev < 0) return hipSuccess;
    int32_t ev = s.read_ev;
    if (ctx->read_gen[ev] != s.read_gen) {
        ev = record_read(ctx, s.read_stream);
        if (ev < 0) return hipErrorUnknown;
    }
    s.read_ev = -1;
    return hipStreamWaitEvent(stream, ctx->read_ring[ev], 0);
}

// Run `launch` on `stream`; with profiling on, give it two events that receive the dispatch's
// begin and end timestamps.
template <typename F>
hipError_t timed_launch(tc_ctx *ctx, int kind, hipStream_t stream, F launch)
{
    if (!ctx->profiling) return launch(Launch{stream, nullptr, nullptr});
    hipEvent_t a = take_event(ctx), b = take_event(ctx);
    if (!a || !b) return hipErrorOutOfMemory;
    hipError_t e = launch(Launch{stream, a, b});
    ctx->timed.push_back(tc_ctx::Timed{kind, a, b});
    return e;
}

bool config_ok(const tc_config *c)
{
    if (!c) return false;
    if (c->n_layers <= 0 || c->n_kv_heads <= 0 || c->n_q_heads <= 0) return false;
    if (c->n_q_heads % c->n_kv_heads != 0) return false;
    if (c->block_size != kBlockTokens) return false;
    if (c->dtype != TC_F32 && c->dtype != TC_BF16) return false;
    if (c->head_dim != 64 && c->head_dim != 128) return false;
    if (c->dtype == TC_BF16 && c->head_dim != 128) return false;
    if (c->table_capacity < 0 || c->max_table_tokens <= 0) return false;
    if (c->policy < TC_POLICY_LRU || c->policy > TC_POLICY_LFU) return false;
    if (c->n_pool_blocks <= 0 || c->n_pool_blocks > INT32_MAX) return false;
    const int64_t sb = (c->max_table_tokens + kBlockTokens - 1) / kBlockTokens;
    if ((int64_t)c->table_capacity * sb > c->n_pool_blocks) return false;
    if (c->slot_layout != TC_SLOTS_ROWS && c->slot_layout != TC_SLOTS_BLOCKS) return false;
    // aliasing sequences: bf16 kernels only; the device block tables keep 5 bits beside the id
    if (c->slot_layout == TC_SLOTS_BLOCKS && (c->dtype != TC_BF16 || c->n_pool_blocks > (int64_t)kBidMask)) return false;
    return true;
}

int esize_of(const tc_config &c) { return c.dtype == TC_F32 ? 4 : 2; }

// Make room for a plan of `ints` integers: the pinned staging buffer on the host and, unless the
// plan goes to the static workspace (`fixed`), the device buffer.  The staging buffer is created
// by tc_create with the static workspace's plan capacity, so a fixed plan never allocates.
tc_status ensure_stage(tc_ctx *ctx, size_t ints, bool fixed)
{
    if (ctx->stage_pending) {                       // the previous upload still reads the staging buffer
        TC_HIP(ctx, hipEventSynchronize(ctx->stage_ev));
        ctx->stage_pending = false;
    }
    if (fixed) {
        if (ints > kScratchPlanInts || ints > ctx->h_stage_ints)
            return fail(ctx, TC_ERR_CAPACITY, "attn (no allocation): the batch's plan needs %zu integers, the fixed workspace holds %zu",
                        ints, std::min(kScratchPlanInts, ctx->h_stage_ints));
        return TC_OK;
    }
    if (ints > ctx->h_stage_ints) {
        if (ctx->h_stage) TC_HIP(ctx, hipHostFree(ctx->h_stage));
        ctx->h_stage = nullptr; ctx->h_stage_ints = 0;
        const size_t cap = std::max(ints * 2, size_t(1) << 16);
        TC_HIP(ctx, hipHostMalloc((void **)&ctx->h_stage, cap * sizeof(int32_t), hipHostMallocDefault));
        ctx->h_stage_ints = cap;
    }
    if (ints > ctx->d_plan_ints) {
        if (ctx->d_plan) TC_HIP(ctx, hipFree(ctx->d_plan));   // hipFree waits for work that may use it
        ctx->d_plan = nullptr; ctx->d_plan_ints = 0;
        const size_t cap = std::max(ints * 2, size_t(1) << 16);
        TC_HIP(ctx, hipMalloc((void **)&ctx->d_plan, cap * sizeof(int32_t)));
        ctx->d_plan_ints = cap;
    }
    return TC_OK;
}

struct SegInfo { int32_t start, len, slot; };

// Serialise the plan into the staging buffer and enqueue its upload on `stream`.
// `fixed`: the device copy and the partials go to the static workspace; nothing is allocated, and a
// batch that does not fit it is refused.
tc_status upload_plan(tc_ctx *ctx, Plan &p, const std::vector<SegInfo> &segs,
                      const std::vector<int32_t> &seg_end_of_q, const std::vector<StitchBlk> &sblk,
                      hipStream_t stream, bool fixed = false)
{
    std::vector<AttnItem> items;
    std::vector<int32_t> splits_of_q;
    std::vector<MergeGroup> groups;
    if (!plan_attention(ctx->cfg, ctx->knobs, p, items, splits_of_q, groups))
        return fail(ctx, TC_ERR_INVALID, "attn: a work item's key range exceeds its kernel's block-id table");

    const size_t B = p.B, nseg = segs.size();
    size_t off = 0;
    auto take = [&](size_t n) { size_t o = off; off += align8(n); return o; };
    const size_t o_bt = take(B * p.max_blocks), o_cu = take(B + 1), o_pl = take(B), o_sl = take(B);
    const size_t o_ss = take(nseg), o_sn = take(nseg), o_st = take(nseg), o_se = take(B);
    const size_t o_sb = take(sblk.size() * 4), o_sp = take(B), o_tq = take(p.total_S);
    const size_t o_it = take(items.size() * (sizeof(AttnItem) / 4));
    const size_t o_gr = take(groups.size() * (sizeof(MergeGroup) / 4));
    const size_t o_rp = take(p.rope ? B : 0), o_rf = take(p.rope ? p.rope_rev_freq.size() * 2 : 0);
    const size_t total = std::max(off, size_t(8));
    // split-KV partials.  bf16 kernels: per (partition, group, row block) 128 rows x (128 fp16 + 2
    // floats) in fragment order, counted in floats; fp32 and decode kernels: per (partition, new
    // token, head) D + 2 floats
    const size_t part_need = !(p.max_splits > 1 || p.decode) ? 0
        : ctx->cfg.dtype == TC_BF16 && !p.decode
            ? (size_t)p.max_splits * p.n_groups * p.row_blocks * kAttnRows * (64 + 2)
            : (size_t)p.max_splits * p.total_S * ctx->cfg.n_q_heads * (ctx->cfg.head_dim + 2);
    if (fixed && part_need > kScratchPartFloats)
        return fail(ctx, TC_ERR_CAPACITY, "attn (no allocation): the split-KV partials need %zu floats, the fixed workspace holds %zu",
                    part_need, kScratchPartFloats);
    tc_status st = ensure_stage(ctx, total, fixed);
    if (st != TC_OK) return st;
    int32_t *h = ctx->h_stage;
    std::memset(h, 0, total * sizeof(int32_t));
    if (B) {
        std::memcpy(h + o_bt, p.block_table.data(), B * p.max_blocks * 4);
        for (size_t k = 0; k < p.block_pad.size(); ++k)
            if (p.block_pad[k]) h[o_bt + k] |= (int32_t)((uint32_t)p.block_pad[k] << kPadShift);
        std::memcpy(h + o_cu, p.cu_seqlens.data(), (B + 1) * 4);
        std::memcpy(h + o_pl, p.prefix_len.data(), B * 4);
        std::memcpy(h + o_sl, p.suffix_len.data(), B * 4);
        std::memcpy(h + o_sp, splits_of_q.data(), B * 4);
        if (!seg_end_of_q.empty()) std::memcpy(h + o_se, seg_end_of_q.data(), B * 4);
    }
    for (size_t k = 0; k < nseg; ++k) {
        h[o_ss + k] = segs[k].start; h[o_sn + k] = segs[k].len; h[o_st + k] = segs[k].slot;
    }
    if (!sblk.empty()) std::memcpy(h + o_sb, sblk.data(), sblk.size() * sizeof(StitchBlk));
    for (int i = 0; i < p.B; ++i)
        for (int n = p.cu_seqlens[i]; n < p.cu_seqlens[i + 1]; ++n) h[o_tq + n] = i;
    if (!items.empty()) std::memcpy(h + o_it, items.data(), items.size() * sizeof(AttnItem));
    if (!groups.empty()) std::memcpy(h + o_gr, groups.data(), groups.size() * sizeof(MergeGroup));
    if (p.rope) {
        if (B) std::memcpy(h + o_rp, p.rope_pos0.data(), B * 4);
        std::memcpy(h + o_rf, p.rope_rev_freq.data(), p.rope_rev_freq.size() * sizeof(double));
    }

    int32_t *d_dst = fixed ? (int32_t *)ctx->scratch_dev : ctx->d_plan;
    TC_HIP(ctx, hipMemcpyAsync(d_dst, h, total * sizeof(int32_t), hipMemcpyHostToDevice, stream));
    TC_HIP(ctx, hipEventRecord(ctx->stage_ev, stream));
    ctx->stage_pending = true;

    const int32_t *d = d_dst;
    p.dev.block_table = d + o_bt; p.dev.cu_seqlens = d + o_cu; p.dev.prefix_len = d + o_pl;
    p.dev.suffix_len = d + o_sl; p.dev.seg_start = d + o_ss; p.dev.seg_len = d + o_sn;
    p.dev.seg_slot = d + o_st; p.dev.seg_end_of_q = d + o_se;
    p.dev.stitch_blk = (const StitchBlk *)(d + o_sb); p.dev.splits_of_q = d + o_sp;
    p.dev.tok_q = d + o_tq;
    p.dev.rope_pos0 = p.rope ? d + o_rp : nullptr;
    p.dev.rope_rev_freq = p.rope ? (const double *)(d + o_rf) : nullptr;
    p.dev.B = p.B; p.dev.max_blocks = p.max_blocks; p.dev.total_S = p.total_S;
    p.dev.n_stitch_blk = (int32_t)sblk.size();
    p.n_stitch_blk = (int32_t)sblk.size();
    p.items_dev = (const AttnItem *)(d + o_it);
    p.groups_dev = (const MergeGroup *)(d + o_gr);

    p.fixed = fixed;
    p.part = nullptr;
    if (fixed) {
        // nothing in the partials has to start at zero: every slot a merge reads was written by the
        // attention launch before it
        if (part_need) p.part = (float *)(ctx->scratch_dev + kScratchPlanInts * 4);
    } else if (part_need) {
        if (part_need > ctx->d_part_floats) {
            if (ctx->d_part) TC_HIP(ctx, hipFree(ctx->d_part));
            ctx->d_part = nullptr; ctx->d_part_floats = 0;
            TC_HIP(ctx, hipMalloc((void **)&ctx->d_part, part_need * sizeof(float)));
            ctx->d_part_floats = part_need;
        }
        p.part = ctx->d_part;
    }
    p.valid = true;
    return TC_OK;
}

}  // namespace

// =========================================================================== C ABI

extern "C" {

size_t tc_block_bytes(const tc_config *c)
{
    if (!c || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->block_size <= 0) return 0;
    return (size_t)2 * c->n_kv_heads * c->block_size * c->head_dim * (c->dtype == TC_F32 ? 4 : 2);
}

size_t tc_pool_bytes(const tc_config *c)
{
    if (!config_ok(c)) return 0;
    size_t blocks = (size_t)c->n_pool_blocks;
    // block-format slots: room for one table as registered (token rows), where a copy from the host
    // lands before it is laid out into the table's slot
    if (c->slot_layout == TC_SLOTS_BLOCKS) blocks += (size_t)((c->max_table_tokens + kBlockTokens - 1) / kBlockTokens);
    return (size_t)c->n_layers * blocks * tc_block_bytes(c);
}

int64_t tc_first_seq_block(const tc_config *c)
{
    if (!config_ok(c)) return -1;
    return (int64_t)c->table_capacity * ((c->max_table_tokens + kBlockTokens - 1) / kBlockTokens);
}

const char *tc_version(void) { return "libtablecache 0.1 (gfx950)"; }

const char *tc_last_error(const tc_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

tc_status tc_create(const tc_config *cfg, void *kv_pool_dev, size_t pool_bytes, tc_ctx **out)
{
    if (!out) return TC_ERR_INVALID;
    *out = nullptr;
    if (!config_ok(cfg) || !kv_pool_dev) return TC_ERR_INVALID;
    if (pool_bytes < tc_pool_bytes(cfg) || ((uintptr_t)kv_pool_dev & 255)) return TC_ERR_INVALID;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev <= 0) return TC_ERR_HIP;   // no CPU fallback exists

    std::unique_ptr<tc_ctx> ctx(new tc_ctx);
    ctx->cfg = *cfg;
    // this device's copy of the static workspace: its address comes from the runtime, once per device,
    // with that device current (the array's name means nothing to host code)
    if (hipGetDevice(&ctx->device) != hipSuccess || ctx->device < 0 || ctx->device >= kMaxDevices) return TC_ERR_HIP;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[ctx->device]) {
            void *ptr = nullptr;
            if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TC_ERR_HIP;
            g_scratch_ptr[ctx->device] = (char *)ptr;
        }
        ctx->scratch_dev = g_scratch_ptr[ctx->device];
    }
    // pinned staging for plan uploads, sized so that a plan bound for the static workspace always fits
    if (hipHostMalloc((void **)&ctx->h_stage, kScratchPlanInts * sizeof(int32_t), hipHostMallocDefault) != hipSuccess)
        return TC_ERR_HIP;
    ctx->h_stage_ints = kScratchPlanInts;
    ctx->slot_blocks = (cfg->max_table_tokens + kBlockTokens - 1) / kBlockTokens;
    ctx->first_seq = tc_first_seq_block(cfg);
    Geom &g = ctx->geom;
    g.block_bytes = (int64_t)tc_block_bytes(cfg);
    g.tab_base = (char *)kv_pool_dev;
    g.slot_bytes = g.block_bytes * ctx->slot_blocks * cfg->n_layers;
    const int64_t n_seq = cfg->n_pool_blocks - ctx->first_seq;
    g.layer_stride = g.block_bytes * n_seq;
    g.pool = (char *)kv_pool_dev + g.slot_bytes * cfg->table_capacity - ctx->first_seq * g.block_bytes;
    if (cfg->slot_layout == TC_SLOTS_BLOCKS) {
        // one block-id space per layer: ids [0, first_seq) are the table slots' blocks (slot s owns
        // s * slot_blocks ..), the rest sequence blocks; the staging area for raw tables follows
        g.pool = (char *)kv_pool_dev;
        g.layer_stride = g.block_bytes * cfg->n_pool_blocks;
        g.tab_base = (char *)kv_pool_dev + g.layer_stride * cfg->n_layers;
    }
    g.first_seq = (int32_t)ctx->first_seq;
    g.n_blocks = (int32_t)cfg->n_pool_blocks;
    g.Hq = cfg->n_q_heads; g.Hkv = cfg->n_kv_heads; g.D = cfg->head_dim; g.G = g.Hq / g.Hkv;
    g.esize = esize_of(*cfg);
    g.row_bytes = g.Hkv * g.D * g.esize;
    g.head_bytes = g.D * g.esize;

    ctx->rule.reset(make_rule(cfg->policy));

    ctx->slots.resize(cfg->table_capacity);
    for (int s = 0; s < cfg->table_capacity; ++s) {
        if (hipEventCreateWithFlags(&ctx->slots[s].ready, hipEventDisableTiming) != hipSuccess) return TC_ERR_HIP;
        ctx->free_slots.insert(s);
    }
    ctx->read_ring.resize(64);
    ctx->read_gen.assign(64, 0);
    for (auto &e : ctx->read_ring)
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return TC_ERR_HIP;
    if (hipEventCreateWithFlags(&ctx->stage_ev, hipEventDisableTiming) != hipSuccess) return TC_ERR_HIP;
    if (hipEventCreateWithFlags(&ctx->raw_ev, hipEventDisableTiming) != hipSuccess) return TC_ERR_HIP;
    ctx->seq.reset(ctx->first_seq, cfg->n_pool_blocks);
    *out = ctx.release();
    return TC_OK;
}

tc_status tc_destroy(tc_ctx *ctx)
{
    if (!ctx) return TC_ERR_INVALID;
    (void)hipDeviceSynchronize();
    for (auto &s : ctx->slots) if (s.ready) (void)hipEventDestroy(s.ready);
    for (auto &e : ctx->read_ring) if (e) (void)hipEventDestroy(e);
    if (ctx->stage_ev) (void)hipEventDestroy(ctx->stage_ev);
    if (ctx->raw_ev) (void)hipEventDestroy(ctx->raw_ev);
    if (ctx->h_stage) (void)hipHostFree(ctx->h_stage);
    if (ctx->d_plan) (void)hipFree(ctx->d_plan);
    if (ctx->d_part) (void)hipFree(ctx->d_part);
    if (ctx->d_read) (void)hipFree(ctx->d_read);
    for (auto &t : ctx->timed) { (void)hipEventDestroy(t.a); (void)hipEventDestroy(t.b); }
    for (auto &e : ctx->ev_pool) (void)hipEventDestroy(e);
    delete ctx;
    return TC_OK;
}

tc_status tc_register_table_kv(tc_ctx *ctx, int32_t table_id, int32_t n_tokens, const void *host_k,
                               const void *host_v)
{
    if (!ctx) return TC_ERR_INVALID;
    if (table_id < 0 || !host_k || !host_v) return fail(ctx, TC_ERR_INVALID, "register: bad id or null KV");
    if (n_tokens <= 0 || n_tokens > ctx->cfg.max_table_tokens)
        return fail(ctx, TC_ERR_CAPACITY, "register: table %d has %d tokens, slot holds %d", table_id,
                    n_tokens, ctx->cfg.max_table_tokens);
    if (ctx->tables.count(table_id)) return fail(ctx, TC_ERR_INVALID, "register: table %d already registered", table_id);
    Table t;
    t.n_tokens = n_tokens;
    t.host_k = (const char *)host_k; t.host_v = (const char *)host_v;
    t.layer_loaded.assign(ctx->cfg.n_layers, 0);
    ctx->tables.emplace(table_id, std::move(t));
    return TC_OK;
}

tc_status tc_load_async(tc_ctx *ctx, const int32_t *table_ids, int32_t n, int32_t l0, int32_t l1, void *stream_)
{
    if (!ctx) return TC_ERR_INVALID;
    if (n < 0 || (n > 0 && !table_ids)) return fail(ctx, TC_ERR_INVALID, "load: bad id list");
    if (l0 < 0 || l1 > ctx->cfg.n_layers || l0 > l1) return fail(ctx, TC_ERR_INVALID, "load: bad layer range [%d,%d)", l0, l1);
    if (ctx->cfg.table_capacity == 0 && n > 0) return fail(ctx, TC_ERR_CAPACITY, "load: table cache has no slots");
    for (int k = 0; k < n; ++k)
        if (!ctx->tables.count(table_ids[k])) return fail(ctx, TC_ERR_UNKNOWN_TABLE, "load: table %d not registered", table_ids[k]);
    hipStream_t stream = (hipStream_t)stream_;
    const Geom &g = ctx->geom;
    // Slots that received copies get their `ready` event recorded behind them on every way out of
    // this call, the early returns included: ids before a failing one stay requested and marked
    // loaded, and whoever reads their slots from another stream must find an event that covers
    // the copies already enqueued.
    struct ReadyGuard {
        tc_ctx *ctx; hipStream_t stream; std::set<int32_t> touched;
        hipError_t flush() {
            hipError_t first = hipSuccess;
            for (int32_t s : touched) {
                Slot &sl = ctx->slots[s];
                const hipError_t e = hipEventRecord(sl.ready, stream);
                if (e != hipSuccess && first == hipSuccess) first = e;
                sl.ready_stream = stream;
                sl.ready_pending = true;
            }
            touched.clear();
            return first;
        }
        ~ReadyGuard() { (void)flush(); }
    } guard{ctx, stream, {}};
    std::set<int32_t> &touched = guard.touched;
    for (int k = 0; k < n; ++k) {
        const int32_t id = table_ids[k];
        Table &t = ctx->tables[id];
        const CacheStep step = cache_request(*ctx->rule, ctx->pins, ctx->cfg.table_capacity, id);
        if (step.refused)
            return fail(ctx, TC_ERR_CAPACITY, "load: table %d needs a slot and all %d cached tables are pinned",
                        id, (int)ctx->cfg.table_capacity);
        const bool hit = step.hit;
        const int32_t evicted = step.evicted;
        if (!hit) {
            if (evicted >= 0) {
                Table &v = ctx->tables[evicted];
                ctx->free_slots.insert(v.slot);
                ctx->slots[v.slot].table = -1;
                v.slot = -1;
                std::fill(v.layer_loaded.begin(), v.layer_loaded.end(), 0);
            }
            t.slot = *ctx->free_slots.begin();
            ctx->free_slots.erase(ctx->free_slots.begin());
            Slot &s = ctx->slots[t.slot];
            s.table = id;
            TC_HIP(ctx, wait_for_reader(ctx, s, stream));   // a stitch may still be reading the previous occupant
            if (s.ready_pending && s.ready_stream != stream)   // earlier copies into this slot on another stream
                TC_HIP(ctx, hipStreamWaitEvent(stream, s.ready, 0));
            if (s.reader_pending) {     // attention launches read the previous occupant in place: wait for
                                        // everything enqueued so far on the stream they run on
                if (s.reader_stream != stream) {
                    const int32_t ev = record_read(ctx, s.reader_stream);
                    if (ev < 0) return fail(ctx, TC_ERR_HIP, "load: hipEventRecord failed");
                    TC_HIP(ctx, hipStreamWaitEvent(stream, ctx->read_ring[ev], 0));
                    for (Slot &o : ctx->slots)      // the same event covers every slot read on that stream
                        if (o.reader_pending && o.reader_stream == s.reader_stream) o.reader_pending = false;
                }
                s.reader_pending = false;
            }
        }
        ctx->trace.push_back(id); ctx->trace.push_back(hit ? 1 : 0); ctx->trace.push_back(evicted);
        // copy the layers of the range that are not on the device yet: a run of consecutive layers of
        // one table is contiguous on both sides, so it goes as two large transfers (K, V); small
        // transfers reach only ~60 % of the link rate
        const size_t width = (size_t)t.n_tokens * g.row_bytes;
        for (int l = l0; l < l1;) {
            if (t.layer_loaded[l]) { ++l; continue; }
            int e = l;
            while (e < l1 && !t.layer_loaded[e]) ++e;
            const bool blocks = ctx->cfg.slot_layout == TC_SLOTS_BLOCKS;
            // block-format slots: the rows land in the staging area (one for all tables; copies and
            // the kernel that lays them out into the slot's blocks are ordered by the stream)
            if (blocks && ctx->raw_pending && ctx->raw_stream != stream)
                TC_HIP(ctx, hipStreamWaitEvent(stream, ctx->raw_ev, 0));
            char *dst = (blocks ? g.tab_base : g.tab_base + (int64_t)t.slot * g.slot_bytes) + (size_t)l * width;
            touched.insert(t.slot);
            TC_HIP(ctx, hipMemcpyAsync(dst, t.host_k + (size_t)l * width, width * (e - l), hipMemcpyHostToDevice, stream));
            TC_HIP(ctx, hipMemcpyAsync(dst + (g.slot_bytes >> 1), t.host_v + (size_t)l * width, width * (e - l),
                                       hipMemcpyHostToDevice, stream));
            if (blocks) {
                TC_HIP(ctx, launch_format(g, g.tab_base, g.slot_bytes >> 1, t.n_tokens, t.slot * ctx->slot_blocks, l, e,
                                          Launch{stream, nullptr, nullptr}));
                TC_HIP(ctx, hipEventRecord(ctx->raw_ev, stream));
                ctx->raw_stream = stream;
                ctx->raw_pending = true;
            }
            for (int x = l; x < e; ++x) t.layer_loaded[x] = 1;
            l = e;
        }
    }
    TC_HIP(ctx, guard.flush());
    return TC_OK;
}

tc_status tc_pin_tables(tc_ctx *ctx, const int32_t *table_ids, int32_t n)
{
    if (!ctx) return TC_ERR_INVALID;
    if (n < 0 || (n > 0 && !table_ids)) return fail(ctx, TC_ERR_INVALID, "pin: bad id list");
    for (int k = 0; k < n; ++k)
        if (!ctx->tables.count(table_ids[k])) return fail(ctx, TC_ERR_UNKNOWN_TABLE, "pin: table %d not registered", table_ids[k]);
    for (int k = 0; k < n; ++k) ctx->pins[table_ids[k]] += 1;
    return TC_OK;
}

tc_status tc_unpin_tables(tc_ctx *ctx, const int32_t *table_ids, int32_t n)
{
    if (!ctx) return TC_ERR_INVALID;
    if (n < 0 || (n > 0 && !table_ids)) return fail(ctx, TC_ERR_INVALID, "unpin: bad id list");
    PinMap left = ctx->pins;           // all or nothing: check the whole list on a copy first
    for (int k = 0; k < n; ++k) {
        auto it = left.find(table_ids[k]);
        if (it == left.end()) return fail(ctx, TC_ERR_INVALID, "unpin: table %d is not pinned (that often)", table_ids[k]);
        if (--it->second == 0) left.erase(it);
    }
    ctx->pins.swap(left);
    return TC_OK;
}

int32_t tc_load_trace(tc_ctx *ctx, int32_t *out, int32_t cap)
{
    if (!ctx || cap < 0 || (cap > 0 && !out)) return TC_ERR_INVALID;
    const int32_t have = (int32_t)(ctx->trace.size() / 3);
    const int32_t n = std::min(have, cap);
    std::memcpy(out, ctx->trace.data(), (size_t)n * 3 * sizeof(int32_t));
    ctx->trace.erase(ctx->trace.begin(), ctx->trace.begin() + (size_t)n * 3);
    return n;
}

int32_t tc_is_resident(const tc_ctx *ctx, int32_t table_id, int32_t l0, int32_t l1)
{
    if (!ctx) return 0;
    auto it = ctx->tables.find(table_id);
    if (it == ctx->tables.end() || it->second.slot < 0) return 0;
    if (l0 < 0 || l1 > ctx->cfg.n_layers || l0 > l1) return 0;
    for (int l = l0; l < l1; ++l) if (!it->second.layer_loaded[l]) return 0;
    return 1;
}

}  // extern "C"

// Common body of tc_stitch_kv and tc_stitch_kv_rope (rope: re-encode the keys by position).
static tc_status stitch_common(tc_ctx *ctx, const int32_t *table_ids, const int32_t *cu_tables, int32_t B,
                               const int32_t *suffix_len, int32_t *block_table, int32_t max_blocks,
                               int32_t *prefix_len, void *stream_, bool rope, const int32_t *pos0,
                               double rope_theta)
{
    if (!ctx) return TC_ERR_INVALID;
    if (ctx->cfg.slot_layout != TC_SLOTS_ROWS)
        return fail(ctx, TC_ERR_INVALID, "stitch: this context keeps tables in block format; use tc_stitch_alias");
    if (B < 0 || max_blocks < 0) return fail(ctx, TC_ERR_INVALID, "stitch: negative size");
    if (B > 0 && (!cu_tables || !suffix_len || !block_table || !prefix_len))
        return fail(ctx, TC_ERR_INVALID, "stitch: null argument");
    if (B > 0 && (cu_tables[0] != 0)) return fail(ctx, TC_ERR_INVALID, "stitch: cu_tables[0] != 0");
    if (rope) {
        if (!(rope_theta > 1.0) || !std::isfinite(rope_theta)) return fail(ctx, TC_ERR_INVALID, "stitch: rope_theta must be finite and > 1");
        if (ctx->cfg.head_dim % (ctx->cfg.dtype == TC_BF16 ? 16 : 8))
            return fail(ctx, TC_ERR_INVALID, "stitch: re-encoding needs head_dim/2 to be a whole number of 16-byte chunks");
        for (int i = 0; pos0 && i < B; ++i)
            if (pos0[i] < 0 || pos0[i] > (1 << 28)) return fail(ctx, TC_ERR_INVALID, "stitch: pos0[%d] out of range", i);
    }
    hipStream_t stream = (hipStream_t)stream_;
    const int L = ctx->cfg.n_layers;

    // ---- validate and size everything before touching any state
    std::vector<SegInfo> segs;
    std::vector<int32_t> seg_end_of_q(B), P(B), need(B);
    int64_t need_total = 0, total_S = 0;
    for (int i = 0; i < B; ++i) {
        if (cu_tables[i + 1] < cu_tables[i]) return fail(ctx, TC_ERR_INVALID, "stitch: cu_tables not monotone");
        if (cu_tables[i + 1] > cu_tables[i] && !table_ids) return fail(ctx, TC_ERR_INVALID, "stitch: null table_ids");
        if (suffix_len[i] < 0) return fail(ctx, TC_ERR_INVALID, "stitch: negative suffix_len");
        int64_t p = 0;
        for (int k = cu_tables[i]; k < cu_tables[i + 1]; ++k) {
            auto it = ctx->tables.find(table_ids[k]);
            if (it == ctx->tables.end()) return fail(ctx, TC_ERR_UNKNOWN_TABLE, "stitch: table %d not registered", table_ids[k]);
            const Table &t = it->second;
            bool all = t.slot >= 0;
            for (int l = 0; all && l < L; ++l) all = t.layer_loaded[l] != 0;
            if (!all) return fail(ctx, TC_ERR_NOT_RESIDENT, "stitch: table %d is not device-resident", table_ids[k]);
            segs.push_back(SegInfo{(int32_t)p, t.n_tokens, t.slot});
            p += t.n_tokens;
            if (p + suffix_len[i] > INT32_MAX / 2) return fail(ctx, TC_ERR_INVALID, "stitch: sequence too long");
        }
        seg_end_of_q[i] = (int32_t)segs.size();
        P[i] = (int32_t)p;
        need[i] = (int32_t)((p + suffix_len[i] + kBlockTokens - 1) / kBlockTokens);
        if (need[i] > max_blocks) return fail(ctx, TC_ERR_OOM_POOL, "stitch: query %d needs %d blocks, max_blocks is %d", i, need[i], max_blocks);
        need_total += need[i];
        total_S += suffix_len[i];
    }
    if (need_total > (int64_t)ctx->seq.n_free())
        return fail(ctx, TC_ERR_OOM_POOL, "stitch: need %lld sequence blocks, %zu free", (long long)need_total, ctx->seq.n_free());
    if (total_S > INT32_MAX / 2) return fail(ctx, TC_ERR_INVALID, "stitch: batch too long");

    // ---- build the plan (host side), then allocate
    Plan p;
    p.B = B; p.max_blocks = max_blocks; p.total_S = (int32_t)total_S;
    p.block_table.assign((size_t)B * max_blocks, -1);
    p.cu_seqlens.assign(B + 1, 0);
    p.prefix_len = P;
    p.suffix_len.assign(suffix_len, suffix_len + B);
    for (int i = 0; i < B; ++i) p.cu_seqlens[i + 1] = p.cu_seqlens[i] + suffix_len[i];
    p.rope = rope;
    if (rope) {
        p.rope_pos0.assign(B, 0);
        if (pos0) p.rope_pos0.assign(pos0, pos0 + B);
        const int D = ctx->cfg.head_dim;
        p.rope_rev_freq.resize(D / 2);
        const double two_pi = 6.283185307179586476925286766559;
        for (int i = 0; i < D / 2; ++i) p.rope_rev_freq[i] = std::pow(rope_theta, -2.0 * i / D) / two_pi;
    }
    const std::vector<int32_t> lowest = ctx->seq.lowest((size_t)need_total);
    auto next_free = lowest.begin();
    std::vector<StitchBlk> sblk;
    for (int i = 0; i < B; ++i) {
        int seg = i ? seg_end_of_q[i - 1] : 0;
        for (int j = 0; j < need[i]; ++j, ++next_free) {
            const int32_t phys = *next_free;
            p.block_table[(size_t)i * max_blocks + j] = phys;
            const int p0 = j * kBlockTokens;
            if (p0 < P[i]) {
                while (p0 >= segs[seg].start + segs[seg].len) ++seg;
                sblk.push_back(StitchBlk{phys, seg, p0, i});
            }
        }
    }
    tc_status st = upload_plan(ctx, p, segs, seg_end_of_q, sblk, stream);
    if (st != TC_OK) return st;               // nothing allocated yet

    // ---- commit: take the blocks, order the gather after the loads it reads, launch
    for (int i = 0; i < B; ++i)
        for (int j = 0; j < need[i]; ++j) ctx->seq.take(p.block_table[(size_t)i * max_blocks + j]);
    std::set<int32_t> used_slots;
    for (const SegInfo &s : segs) used_slots.insert(s.slot);
    for (int32_t s : used_slots) {
        Slot &sl = ctx->slots[s];
        if (sl.ready_pending && sl.ready_stream != stream)
            TC_HIP(ctx, hipStreamWaitEvent(stream, sl.ready, 0));
    }
    ctx->plan = std::move(p);
    TC_HIP(ctx, timed_launch(ctx, 0, stream, [&](const Launch &ln) { return launch_stitch(ctx->geom, ctx->plan.dev, 0, L, ctx->plan.rope, ln); }));
    if (!used_slots.empty()) {
        const int32_t ev = record_read(ctx, stream);
        if (ev < 0) return fail(ctx, TC_ERR_HIP, "stitch: hipEventRecord failed");
        for (int32_t s : used_slots) {
            Slot &sl = ctx->slots[s];
            sl.read_ev = ev; sl.read_gen = ctx->read_gen[ev]; sl.read_stream = stream;
        }
    }
    if (B > 0) {
        std::memcpy(block_table, ctx->plan.block_table.data(), (size_t)B * max_blocks * sizeof(int32_t));
        std::memcpy(prefix_len, ctx->plan.prefix_len.data(), (size_t)B * sizeof(int32_t));
    }
    return TC_OK;
}

extern "C" {

tc_status tc_stitch_kv(tc_ctx *ctx, const int32_t *table_ids, const int32_t *cu_tables, int32_t B,
                       const int32_t *suffix_len, int32_t *block_table, int32_t max_blocks,
                       int32_t *prefix_len, void *stream)
{
    return stitch_common(ctx, table_ids, cu_tables, B, suffix_len, block_table, max_blocks, prefix_len, stream,
                         false, nullptr, 0.0);
}

tc_status tc_stitch_kv_rope(tc_ctx *ctx, const int32_t *table_ids, const int32_t *cu_tables, int32_t B,
                            const int32_t *suffix_len, const int32_t *pos0, double rope_theta,
                            int32_t *block_table, int32_t max_blocks, int32_t *prefix_len, void *stream)
{
    return stitch_common(ctx, table_ids, cu_tables, B, suffix_len, block_table, max_blocks, prefix_len, stream,
                         true, pos0, rope_theta);
}

// Block-format slots: the number of unused token positions of block id `b` of a table slot, or -1
// if no fully loaded table covers that block.
static int32_t slot_block_pad(const tc_ctx *ctx, int32_t b)
{
    const int32_t s = b / ctx->slot_blocks, j = b % ctx->slot_blocks;
    if (s < 0 || s >= (int32_t)ctx->slots.size() || ctx->slots[s].table < 0) return -1;
    auto it = ctx->tables.find(ctx->slots[s].table);
    if (it == ctx->tables.end()) return -1;
    const Table &t = it->second;
    for (uint8_t l : t.layer_loaded) if (!l) return -1;
    const int nb = (t.n_tokens + kBlockTokens - 1) / kBlockTokens;
    if (j >= nb) return -1;
    return j == nb - 1 ? nb * kBlockTokens - t.n_tokens : 0;
}

tc_status tc_stitch_alias(tc_ctx *ctx, const int32_t *table_ids, const int32_t *cu_tables, int32_t B,
                          const int32_t *suffix_len, int32_t *block_table, int32_t max_blocks,
                          int32_t *prefix_len, void *stream_)
{
    if (!ctx) return TC_ERR_INVALID;
    if (ctx->cfg.slot_layout != TC_SLOTS_BLOCKS)
        return fail(ctx, TC_ERR_INVALID, "alias: this context keeps tables as token rows; use tc_stitch_kv");
    if (B < 0 || max_blocks < 0) return fail(ctx, TC_ERR_INVALID, "alias: negative size");
    if (B > 0 && (!cu_tables || !suffix_len || !block_table || !prefix_len))
        return fail(ctx, TC_ERR_INVALID, "alias: null argument");
    if (B > 0 && (cu_tables[0] != 0)) return fail(ctx, TC_ERR_INVALID, "alias: cu_tables[0] != 0");
    hipStream_t stream = (hipStream_t)stream_;
    const int L = ctx->cfg.n_layers;

    // ---- validate and size everything before touching any state
    std::vector<int32_t> n_pref(B), n_suf(B);
    int64_t need_total = 0, total_S = 0;
    for (int i = 0; i < B; ++i) {
        if (cu_tables[i + 1] < cu_tables[i]) return fail(ctx, TC_ERR_INVALID, "alias: cu_tables not monotone");
        if (cu_tables[i + 1] > cu_tables[i] && !table_ids) return fail(ctx, TC_ERR_INVALID, "alias: null table_ids");
        if (suffix_len[i] < 0) return fail(ctx, TC_ERR_INVALID, "alias: negative suffix_len");
        int64_t nb = 0;
        for (int k = cu_tables[i]; k < cu_tables[i + 1]; ++k) {
            auto it = ctx->tables.find(table_ids[k]);
            if (it == ctx->tables.end()) return fail(ctx, TC_ERR_UNKNOWN_TABLE, "alias: table %d not registered", table_ids[k]);
            const Table &t = it->second;
            bool all = t.slot >= 0;
            for (int l = 0; all && l < L; ++l) all = t.layer_loaded[l] != 0;
            if (!all) return fail(ctx, TC_ERR_NOT_RESIDENT, "alias: table %d is not device-resident", table_ids[k]);
            nb += (t.n_tokens + kBlockTokens - 1) / kBlockTokens;
            if (nb * kBlockTokens + suffix_len[i] > INT32_MAX / 2) return fail(ctx, TC_ERR_INVALID, "alias: sequence too long");
        }
        n_pref[i] = (int32_t)nb;
        n_suf[i] = (suffix_len[i] + kBlockTokens - 1) / kBlockTokens;
        if (nb + n_suf[i] > max_blocks)
            return fail(ctx, TC_ERR_OOM_POOL, "alias: query %d needs %lld blocks, max_blocks is %d", i, (long long)(nb + n_suf[i]), max_blocks);
        need_total += n_suf[i];
        total_S += suffix_len[i];
    }
    if (need_total > (int64_t)ctx->seq.n_free())
        return fail(ctx, TC_ERR_OOM_POOL, "alias: need %lld sequence blocks, %zu free", (long long)need_total, ctx->seq.n_free());
    if (total_S > INT32_MAX / 2) return fail(ctx, TC_ERR_INVALID, "alias: batch too long");

    // ---- the plan: each table contributes the blocks of its slot, the suffix gets blocks of its own
    Plan p;
    p.B = B; p.max_blocks = max_blocks; p.total_S = (int32_t)total_S;
    p.block_table.assign((size_t)B * max_blocks, -1);
    p.block_pad.assign((size_t)B * max_blocks, 0);
    p.cu_seqlens.assign(B + 1, 0);
    p.prefix_len.assign(B, 0);
    p.suffix_len.assign(suffix_len, suffix_len + B);
    std::set<int32_t> used_slots;
    const std::vector<int32_t> lowest = ctx->seq.lowest((size_t)need_total);
    auto next_free = lowest.begin();
    for (int i = 0; i < B; ++i) {
        p.cu_seqlens[i + 1] = p.cu_seqlens[i] + suffix_len[i];
        p.prefix_len[i] = n_pref[i] * kBlockTokens;
        size_t at = (size_t)i * max_blocks;
        for (int k = cu_tables[i]; k < cu_tables[i + 1]; ++k) {
            const Table &t = ctx->tables[table_ids[k]];
            const int nb = (t.n_tokens + kBlockTokens - 1) / kBlockTokens;
            for (int j = 0; j < nb; ++j, ++at) p.block_table[at] = t.slot * ctx->slot_blocks + j;
            p.block_pad[at - 1] = (uint8_t)(nb * kBlockTokens - t.n_tokens);
            used_slots.insert(t.slot);
        }
        for (int j = 0; j < n_suf[i]; ++j, ++next_free, ++at) p.block_table[at] = *next_free;
    }
    p.alias_slots.assign(used_slots.begin(), used_slots.end());
    tc_status st = upload_plan(ctx, p, {}, {}, {}, stream);
    if (st != TC_OK) return st;               // nothing allocated yet

    // ---- commit: take the suffix blocks; whatever follows on `stream` comes after the loads it reads
    for (int i = 0; i < B; ++i)
        for (int j = n_pref[i]; j < n_pref[i] + n_suf[i]; ++j) ctx->seq.take(p.block_table[(size_t)i * max_blocks + j]);
    for (int32_t s : used_slots) {
        Slot &sl = ctx->slots[s];
        if (sl.ready_pending && sl.ready_stream != stream)
            TC_HIP(ctx, hipStreamWaitEvent(stream, sl.ready, 0));
        sl.reader_stream = stream;
        sl.reader_pending = true;
    }
    ctx->plan = std::move(p);
    if (B > 0) {
        std::memcpy(block_table, ctx->plan.block_table.data(), (size_t)B * max_blocks * sizeof(int32_t));
        std::memcpy(prefix_len, ctx->plan.prefix_len.data(), (size_t)B * sizeof(int32_t));
    }
    return TC_OK;
}

}  // extern "C"

// Common body of tc_prefill_attn and tc_prefill_attn_noalloc (`fixed`: plan and partials in the static
// workspace, no allocation on the way).
static tc_status prefill_common(tc_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new,
                                void *out, const int32_t *cu_seqlens, const int32_t *block_table,
                                int32_t max_blocks, const int32_t *prefix_len, const int32_t *suffix_len,
                                int32_t B, float sm_scale, void *stream_, bool fixed)
{
    if (!ctx) return TC_ERR_INVALID;
    if (layer < 0 || layer >= ctx->cfg.n_layers) return fail(ctx, TC_ERR_INVALID, "attn: layer %d out of range", layer);
    if (B < 0 || max_blocks < 0) return fail(ctx, TC_ERR_INVALID, "attn: negative size");
    if (!(sm_scale > 0.f) || !std::isfinite(sm_scale)) return fail(ctx, TC_ERR_INVALID, "attn: sm_scale must be positive and finite");
    if (B == 0) return TC_OK;
    if (!cu_seqlens || !block_table || !prefix_len || !suffix_len) return fail(ctx, TC_ERR_INVALID, "attn: null integer argument");
    hipStream_t stream = (hipStream_t)stream_;
    Plan &cur = ctx->plan;
    const bool same = cur.valid && cur.fixed == fixed && cur.B == B && cur.max_blocks == max_blocks &&
                      !std::memcmp(cur.cu_seqlens.data(), cu_seqlens, (size_t)(B + 1) * 4) &&
                      !std::memcmp(cur.prefix_len.data(), prefix_len, (size_t)B * 4) &&
                      !std::memcmp(cur.suffix_len.data(), suffix_len, (size_t)B * 4) &&
                      !std::memcmp(cur.block_table.data(), block_table, (size_t)B * max_blocks * 4);
    if (!same) {
        // a caller-made batch: check every integer the kernels will index with, then plan it
        if (cu_seqlens[0] != 0) return fail(ctx, TC_ERR_INVALID, "attn: cu_seqlens[0] != 0");
        Plan p;
        p.B = B; p.max_blocks = max_blocks;
        std::set<int32_t> used_slots;
        for (int i = 0; i < B; ++i) {
            if (prefix_len[i] < 0 || suffix_len[i] < 0 || cu_seqlens[i + 1] - cu_seqlens[i] != suffix_len[i])
                return fail(ctx, TC_ERR_INVALID, "attn: lengths of query %d are inconsistent", i);
            const int64_t nb = ((int64_t)prefix_len[i] + suffix_len[i] + kBlockTokens - 1) / kBlockTokens;
            if (nb > max_blocks) return fail(ctx, TC_ERR_INVALID, "attn: query %d needs %lld blocks > max_blocks", i, (long long)nb);
            for (int j = 0; j < nb; ++j) {
                const int32_t b = block_table[(size_t)i * max_blocks + j];
                if (b >= ctx->first_seq && b < ctx->cfg.n_pool_blocks) continue;
                // block-format slots: a block of a cached table, read in place.  Which of its
                // positions hold tokens follows from the table that sits in the slot now.
                int32_t pad = -1;
                if (ctx->cfg.slot_layout == TC_SLOTS_BLOCKS && b >= 0 && b < ctx->first_seq &&
                    (int64_t)(j + 1) * kBlockTokens <= prefix_len[i])
                    pad = slot_block_pad(ctx, b);
                if (pad < 0)
                    return fail(ctx, TC_ERR_INVALID, "attn: block_table[%d][%d] = %d is not a block this sequence may read", i, j, b);
                if (p.block_pad.empty()) p.block_pad.assign((size_t)B * max_blocks, 0);
                p.block_pad[(size_t)i * max_blocks + j] = (uint8_t)pad;
                used_slots.insert(b / ctx->slot_blocks);
            }
        }
        p.alias_slots.assign(used_slots.begin(), used_slots.end());
        p.total_S = cu_seqlens[B];
        p.block_table.assign(block_table, block_table + (size_t)B * max_blocks);
        p.cu_seqlens.assign(cu_seqlens, cu_seqlens + B + 1);
        p.prefix_len.assign(prefix_len, prefix_len + B);
        p.suffix_len.assign(suffix_len, suffix_len + B);
        tc_status st = upload_plan(ctx, p, {}, {}, {}, stream, fixed);
        if (st != TC_OK) return st;
        for (int32_t sidx : p.alias_slots) {        // the launches come after the loads of what they read
            Slot &sl = ctx->slots[sidx];
            if (sl.ready_pending && sl.ready_stream != stream) TC_HIP(ctx, hipStreamWaitEvent(stream, sl.ready, 0));
        }
        ctx->plan = std::move(p);
    }
    Plan &p = ctx->plan;
    if (p.total_S == 0) return TC_OK;
    if (!q || !k_new || !v_new || !out) return fail(ctx, TC_ERR_INVALID, "attn: null tensor");
    for (int32_t sidx : p.alias_slots) {        // this launch reads these table slots in place
        ctx->slots[sidx].reader_stream = stream;
        ctx->slots[sidx].reader_pending = true;
    }
    if (((uintptr_t)q | (uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)out) & 15)
        return fail(ctx, TC_ERR_INVALID, "attn: tensors must be 16-byte aligned");

    const bool bf16 = ctx->cfg.dtype == TC_BF16;
    if (p.decode) {
        AttnArgs a{};
        a.q = q; a.k_new = k_new; a.v_new = v_new; a.out = out;
        a.n_append = p.total_S + p.B; a.items = p.items_dev; a.n_items = p.n_items; a.layer = layer;
        a.scale_log2 = sm_scale * 1.4426950408889634f;
        a.part_o = p.part;
        a.part_ml = p.part + (size_t)p.max_splits * p.total_S * ctx->cfg.n_q_heads * ctx->cfg.head_dim;
        TC_HIP(ctx, timed_launch(ctx, 2, stream, [&](const Launch &ln) { return launch_decode_bf16(ctx->geom, p.dev, a, ln); }));
        TC_HIP(ctx, timed_launch(ctx, 3, stream, [&](const Launch &ln) { return launch_decode_finish(ctx->geom, p.dev, a, p.max_splits, ln); }));
        return TC_OK;
    }
    if (!bf16)      // the bf16 attention launches append in extra work-groups of their own, except:
        TC_HIP(ctx, timed_launch(ctx, 1, stream, [&](const Launch &ln) { return launch_append(ctx->geom, p.dev, layer, k_new, v_new, ln); }));
    if (p.pingpong) {   // this kernel reads the suffix from the pool: it is appended first, block by block
        int n_blk = 0;
        for (int i = 0; i < p.B; ++i)
            if (p.suffix_len[i] > 0)
                n_blk += (p.prefix_len[i] + p.suffix_len[i] + kBlockTokens - 1) / kBlockTokens - p.prefix_len[i] / kBlockTokens;
        TC_HIP(ctx, timed_launch(ctx, 1, stream, [&](const Launch &ln) { return launch_append_blocks(ctx->geom, p.dev, layer, k_new, v_new, n_blk, ln); }));
    }
    AttnArgs a{};
    a.q = q; a.k_new = k_new; a.v_new = v_new; a.out = out;
    a.n_append = bf16 && !p.pingpong ? p.total_S + p.B : 0; a.items = p.items_dev; a.n_items = p.n_items; a.layer = layer;
    a.scale_log2 = sm_scale * 1.4426950408889634f;
    a.has_pads = p.block_pad.empty() ? 0 : 1;
    a.part_o = p.part;
    a.part_ml = !p.part ? nullptr
              : bf16 ? p.part + (size_t)p.max_splits * p.n_groups * p.row_blocks * kAttnRows * 64
                     : p.part + (size_t)p.max_splits * p.total_S * ctx->cfg.n_q_heads * ctx->cfg.head_dim;
    TC_HIP(ctx, timed_launch(ctx, 2, stream, [&](const Launch &ln) {
        return p.pingpong ? launch_attn_pp_bf16(ctx->geom, p.dev, a, ln)
             : bf16 ? launch_attn_bf16(ctx->geom, p.dev, a, p.row_blocks, p.pipelined, ln)
                    : launch_attn_f32(ctx->geom, p.dev, a, ln);
    }));
    if (p.max_splits > 1)
        TC_HIP(ctx, timed_launch(ctx, 3, stream, [&](const Launch &ln) {
            return bf16 ? launch_merge_bf16(ctx->geom, a, p.groups_dev, p.n_groups, p.row_blocks, ln)
                        : launch_merge(ctx->geom, p.dev, a, ln);
        }));
    return TC_OK;
}

extern "C" {

tc_status tc_prefill_attn(tc_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new,
                          void *out, const int32_t *cu_seqlens, const int32_t *block_table,
                          int32_t max_blocks, const int32_t *prefix_len, const int32_t *suffix_len,
                          int32_t B, float sm_scale, void *stream)
{
    return prefill_common(ctx, layer, q, k_new, v_new, out, cu_seqlens, block_table, max_blocks, prefix_len,
                          suffix_len, B, sm_scale, stream, false);
}

tc_status tc_prefill_attn_noalloc(tc_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new,
                                  void *out, const int32_t *cu_seqlens, const int32_t *block_table,
                                  int32_t max_blocks, const int32_t *prefix_len, const int32_t *suffix_len,
                                  int32_t B, float sm_scale, void *stream)
{
    if (ctx && !ctx->scratch_dev) return fail(ctx, TC_ERR_HIP, "attn (no allocation): the static workspace was not resolved");
    return prefill_common(ctx, layer, q, k_new, v_new, out, cu_seqlens, block_table, max_blocks, prefix_len,
                          suffix_len, B, sm_scale, stream, true);
}

tc_status tc_grow_seqs(tc_ctx *ctx, int32_t *block_table, int32_t max_blocks, int32_t B, const int32_t *new_len)
{
    if (!ctx) return TC_ERR_INVALID;
    if (B < 0 || max_blocks < 0 || (B > 0 && (!block_table || !new_len)))
        return fail(ctx, TC_ERR_INVALID, "grow: bad arguments");
    // size first, change nothing on failure
    std::vector<int32_t> have(B), want(B);
    int64_t need_total = 0;
    for (int i = 0; i < B; ++i) {
        if (new_len[i] < 0) return fail(ctx, TC_ERR_INVALID, "grow: negative length");
        const int32_t *row = block_table + (size_t)i * max_blocks;
        int h = 0;
        while (h < max_blocks && row[h] >= 0) {
            const bool table_block = ctx->cfg.slot_layout == TC_SLOTS_BLOCKS && row[h] < ctx->first_seq;   // read in place
            if (!table_block && !ctx->seq.allocated(row[h]))
                return fail(ctx, TC_ERR_INVALID, "grow: %d is not an allocated sequence block", row[h]);
            ++h;
        }
        have[i] = h;
        want[i] = (int32_t)(((int64_t)new_len[i] + kBlockTokens - 1) / kBlockTokens);
        if (want[i] > max_blocks)
            return fail(ctx, TC_ERR_OOM_POOL, "grow: query %d needs %d blocks, max_blocks is %d", i, want[i], max_blocks);
        if (want[i] > h) need_total += want[i] - h;
    }
    if (need_total > (int64_t)ctx->seq.n_free())
        return fail(ctx, TC_ERR_OOM_POOL, "grow: need %lld sequence blocks, %zu free", (long long)need_total, ctx->seq.n_free());
    for (int i = 0; i < B; ++i)
        for (int j = have[i]; j < want[i]; ++j) block_table[(size_t)i * max_blocks + j] = ctx->seq.take_lowest();
    return TC_OK;
}

tc_status tc_release_seqs(tc_ctx *ctx, const int32_t *block_table, int32_t max_blocks, int32_t B)
{
    if (!ctx) return TC_ERR_INVALID;
    if (B < 0 || max_blocks < 0 || ((int64_t)B * max_blocks > 0 && !block_table))
        return fail(ctx, TC_ERR_INVALID, "release: bad arguments");
    const size_t n = (size_t)B * max_blocks;
    std::set<int32_t> seen;
    for (size_t k = 0; k < n; ++k) {
        const int32_t b = block_table[k];
        if (b < 0) continue;
        if (ctx->cfg.slot_layout == TC_SLOTS_BLOCKS && b < ctx->first_seq) continue;   // a table slot's block, aliased
        if (!ctx->seq.allocated(b) || !seen.insert(b).second)
            return fail(ctx, TC_ERR_INVALID, "release: %d is not an allocated sequence block", b);
    }
    for (int32_t b : seen) ctx->seq.release(b);
    if (ctx->plan.valid && (!seen.empty() || !ctx->plan.alias_slots.empty()))
        ctx->plan.valid = false;               // its blocks may be handed out again
    return TC_OK;
}

tc_status tc_read_seq_kv(tc_ctx *ctx, int32_t layer, const int32_t *blocks, int32_t n_tokens, void *out_k,
                         void *out_v, void *stream_)
{
    if (!ctx) return TC_ERR_INVALID;
    if (layer < 0 || layer >= ctx->cfg.n_layers || n_tokens < 0) return fail(ctx, TC_ERR_INVALID, "read: bad layer or length");
    if (n_tokens == 0) return TC_OK;
    if (!blocks || !out_k || !out_v) return fail(ctx, TC_ERR_INVALID, "read: null argument");
    const int nb = (n_tokens + kBlockTokens - 1) / kBlockTokens;
    for (int j = 0; j < nb; ++j)
        if (blocks[j] < (ctx->cfg.slot_layout == TC_SLOTS_BLOCKS ? 0 : ctx->first_seq) || blocks[j] >= ctx->cfg.n_pool_blocks)
            return fail(ctx, TC_ERR_INVALID, "read: block %d is not a sequence block", blocks[j]);
    hipStream_t stream = (hipStream_t)stream_;
    const size_t bytes = (size_t)n_tokens * ctx->geom.row_bytes;
    const size_t ids_at = (2 * bytes + 255) & ~size_t(255), need = ids_at + (size_t)nb * sizeof(int32_t);
    if (need > ctx->d_read_bytes) {                  // one staging buffer, kept and grown on demand
        if (ctx->d_read) TC_HIP(ctx, hipFree(ctx->d_read));
        ctx->d_read = nullptr; ctx->d_read_bytes = 0;
        TC_HIP(ctx, hipMalloc((void **)&ctx->d_read, need * 2));
        ctx->d_read_bytes = need * 2;
    }
    char *d_k = ctx->d_read, *d_v = ctx->d_read + bytes;
    int32_t *d_b = (int32_t *)(ctx->d_read + ids_at);
    tc_status st = TC_OK;
    hipError_t e = hipMemcpyAsync(d_b, blocks, nb * sizeof(int32_t), hipMemcpyHostToDevice, stream);
    if (e == hipSuccess) e = launch_readback(ctx->geom, layer, d_b, n_tokens, d_k, d_v, stream);
    if (e == hipSuccess) e = hipMemcpyAsync(out_k, d_k, bytes, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipMemcpyAsync(out_v, d_v, bytes, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) st = fail(ctx, TC_ERR_HIP, "read: %s", hipGetErrorString(e));
    return st;
}

tc_status tc_profile_enable(tc_ctx *ctx, int32_t on)
{
    if (!ctx) return TC_ERR_INVALID;
    ctx->profiling = on != 0;
    return TC_OK;
}

tc_status tc_profile_read(tc_ctx *ctx, double *ms_out, int64_t *count_out)
{
    if (!ctx || !ms_out || !count_out) return TC_ERR_INVALID;
    for (auto &t : ctx->timed) {
        float ms = 0.f;
        TC_HIP(ctx, hipEventSynchronize(t.b));
        TC_HIP(ctx, hipEventElapsedTime(&ms, t.a, t.b));
        ctx->prof_ms[t.kind] += ms;
        ctx->prof_n[t.kind] += 1;
        ctx->ev_pool.push_back(t.a); ctx->ev_pool.push_back(t.b);
    }
    ctx->timed.clear();
    for (int k = 0; k < 4; ++k) {
        ms_out[k] = ctx->prof_ms[k]; count_out[k] = ctx->prof_n[k];
        ctx->prof_ms[k] = 0; ctx->prof_n[k] = 0;
    }
    return TC_OK;
}

int32_t tc_kv_splits(const tc_ctx *ctx) { return (ctx && ctx->plan.valid) ? ctx->plan.max_splits : 1; }

tc_status tc_set_kv_splits(tc_ctx *ctx, int32_t n_splits)
{
    if (!ctx || n_splits < 0) return TC_ERR_INVALID;
    ctx->knobs.forced_splits = n_splits;
    ctx->plan.valid = false;
    return TC_OK;
}

int32_t tc_attn_kernel(const tc_ctx *ctx)
{
    if (!ctx || !ctx->plan.valid || ctx->cfg.dtype != TC_BF16) return 0;
    if (ctx->plan.decode) return 3;
    if (ctx->plan.pingpong) return 4;
    if (ctx->plan.row_blocks != 1) return 0;
    return ctx->plan.pipelined ? 2 : 1;
}

tc_status tc_set_attn_kernel(tc_ctx *ctx, int32_t kind)
{
    if (!ctx || kind < 0 || kind > 4) return TC_ERR_INVALID;
    ctx->knobs.forced_attn_kernel = kind;
    ctx->plan.valid = false;
    return TC_OK;
}

tc_status tc_set_row_blocks(tc_ctx *ctx, int32_t row_blocks)
{
    if (!ctx || row_blocks < 0 || row_blocks > 2) return TC_ERR_INVALID;
    ctx->knobs.forced_row_blocks = row_blocks;
    ctx->plan.valid = false;
    return TC_OK;
}

}  // extern "C"
