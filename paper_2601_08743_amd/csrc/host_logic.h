// Host-only logic of libtablecache, free of the HIP headers so that it also builds with a plain C++
// compiler (the sanitizer build of tests/test_host_sanitized.py): the replacement rules of the
// device table cache (paper App. A), the allocator of sequence blocks, and the planner that turns a
// batch into attention work items.  tc_host.hip is the only user in the library.
#pragma once
#include "../../include/tablecache.h"
#include "tc_types.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <list>
#include <set>
#include <unordered_map>
#include <vector>

namespace tc {

// ------------------------------------------------------------------ replacement rules (App. A)
// Each rule answers three questions about the set of cached tables: is the request cached,
// what happens on a hit, and who goes when a miss finds the cache full.  Tables a caller has
// pinned are passed over: the victim is the rule's first choice among the others (-1: none left).
using PinMap = std::unordered_map<int32_t, int32_t>;

class Replacement {
public:
    virtual ~Replacement() {}
    virtual bool cached(int32_t id) const = 0;
    virtual void on_hit(int32_t id) = 0;
    virtual int32_t pick_victim(const PinMap &pins) const = 0;
    virtual void remove(int32_t id) = 0;
    virtual void insert(int32_t id) = 0;
    virtual size_t size() const = 0;
    virtual void tick() {}                         // called once per request, before anything else
};

// LRU: recency list, most recent at the front; the end is evicted.
class LruRule : public Replacement {
    std::list<int32_t> order_;
    std::unordered_map<int32_t, std::list<int32_t>::iterator> pos_;
public:
    bool cached(int32_t id) const override { return pos_.count(id) != 0; }
    void on_hit(int32_t id) override { order_.splice(order_.begin(), order_, pos_[id]); }
    int32_t pick_victim(const PinMap &pins) const override {
        for (auto it = order_.rbegin(); it != order_.rend(); ++it) if (!pins.count(*it)) return *it;
        return -1;
    }
    void remove(int32_t id) override { order_.erase(pos_[id]); pos_.erase(id); }
    void insert(int32_t id) override { order_.push_front(id); pos_[id] = order_.begin(); }
    size_t size() const override { return pos_.size(); }
};

// FIFO: a queue; hits leave it alone; the head is evicted, arrivals join the tail.
class FifoRule : public Replacement {
    std::list<int32_t> queue_;
    std::unordered_map<int32_t, std::list<int32_t>::iterator> pos_;
public:
    bool cached(int32_t id) const override { return pos_.count(id) != 0; }
    void on_hit(int32_t) override {}
    int32_t pick_victim(const PinMap &pins) const override {
        for (int32_t id : queue_) if (!pins.count(id)) return id;
        return -1;
    }
    void remove(int32_t id) override { queue_.erase(pos_[id]); pos_.erase(id); }
    void insert(int32_t id) override { queue_.push_back(id); pos_[id] = std::prev(queue_.end()); }
    size_t size() const override { return pos_.size(); }
};

// LFU: (frequency, timestamp) per table; smallest frequency goes, ties by smallest timestamp.
class LfuRule : public Replacement {
    struct Stat { int64_t freq, stamp; };
    std::unordered_map<int32_t, Stat> stat_;
    int64_t clock_ = 0;
public:
    void tick() override { ++clock_; }
    bool cached(int32_t id) const override { return stat_.count(id) != 0; }
    void on_hit(int32_t id) override { Stat &s = stat_[id]; s.freq += 1; s.stamp = clock_; }
    int32_t pick_victim(const PinMap &pins) const override {
        int32_t best = -1; Stat bs{0, 0};
        for (const auto &kv : stat_)
            if (pins.count(kv.first)) continue;
            else if (best < 0 || kv.second.freq < bs.freq ||
                (kv.second.freq == bs.freq && kv.second.stamp < bs.stamp)) { best = kv.first; bs = kv.second; }
        return best;
    }
    void remove(int32_t id) override { stat_.erase(id); }
    void insert(int32_t id) override { stat_[id] = Stat{1, clock_}; }
    size_t size() const override { return stat_.size(); }
};

// One request against the cache (App. A's Update(request), with pinned tables passed over): a hit
// updates the rule's bookkeeping; a miss on a full cache removes the rule's first unpinned choice
// and inserts the request.  `refused`: a miss found every cached table pinned - nothing changed
// beyond the rule's clock.
struct CacheStep { bool hit; int32_t evicted; bool refused; };
inline CacheStep cache_request(Replacement &rule, const PinMap &pins, int64_t capacity, int32_t id)
{
    rule.tick();
    if (rule.cached(id)) { rule.on_hit(id); return CacheStep{true, -1, false}; }
    int32_t evicted = -1;
    if ((int64_t)rule.size() >= capacity) {
        evicted = rule.pick_victim(pins);
        if (evicted < 0) return CacheStep{false, -1, true};
        rule.remove(evicted);
    }
    rule.insert(id);
    return CacheStep{false, evicted, false};
}

inline Replacement *make_rule(int32_t policy)
{
    if (policy == TC_POLICY_LRU) return new LruRule;
    if (policy == TC_POLICY_FIFO) return new FifoRule;
    return new LfuRule;
}

// ------------------------------------------------------------------ sequence blocks
// Blocks [first, end) of the pool belong to sequences.  Allocation always takes the lowest-numbered
// free block (the paper has no allocator; this rule makes block tables reproducible).
class SeqBlocks {
    int64_t first_ = 0, end_ = 0;
    std::set<int32_t> free_;
    std::vector<uint8_t> used_;
public:
    void reset(int64_t first, int64_t end)
    {
        first_ = first; end_ = end;
        free_.clear();
        for (int64_t b = first; b < end; ++b) free_.insert((int32_t)b);
        used_.assign((size_t)(end - first), 0);
    }
    size_t n_free() const { return free_.size(); }
    bool in_range(int64_t b) const { return b >= first_ && b < end_; }
    bool allocated(int64_t b) const { return in_range(b) && used_[(size_t)(b - first_)] != 0; }
    // the n lowest free blocks in ascending order, not taken yet (n <= n_free())
    std::vector<int32_t> lowest(size_t n) const
    {
        std::vector<int32_t> out;
        out.reserve(n);
        for (auto it = free_.begin(); it != free_.end() && out.size() < n; ++it) out.push_back(*it);
        return out;
    }
    void take(int32_t b) { free_.erase(b); used_[(size_t)(b - first_)] = 1; }
    int32_t take_lowest() { const int32_t b = *free_.begin(); take(b); return b; }
    void release(int32_t b) { used_[(size_t)(b - first_)] = 0; free_.insert(b); }
};

// ------------------------------------------------------------------ the plan of one batch
// The integer plan of one batch, host copy and layout of the device copy.
struct Plan {
    bool valid = false;
    int32_t B = 0, max_blocks = 0, total_S = 0, n_stitch_blk = 0, n_items = 0, max_splits = 1, n_groups = 0, row_blocks = 1;
    bool pipelined = false;     // bf16, one row block per wave: the pipelined attention kernel
    bool decode = false;        // bf16, at most one new token per query: the decode kernels
    bool pingpong = false;      // bf16, 256 rows per work-group in two alternating wave groups; the suffix is appended first
    bool rope = false;          // the stitch re-encodes keys by position (Sec. 4.1.1)
    std::vector<int32_t> rope_pos0;      // [B]
    std::vector<double> rope_rev_freq;   // [D/2]
    std::vector<int32_t> block_table, cu_seqlens, prefix_len, suffix_len;
    std::vector<uint8_t> block_pad;      // aliasing sequences: unused token positions per block-table entry, else empty
    std::vector<int32_t> alias_slots;    // table slots whose blocks the batch's sequences alias
    bool fixed = false;         // plan and partials live in the static workspace (tc_prefill_attn_noalloc)
    float *part = nullptr;      // split-KV partials of this plan (null: none needed)
    BatchDev dev{};
    const AttnItem *items_dev = nullptr;
    const MergeGroup *groups_dev = nullptr;
};

// What a caller may force about the attention launch (tc_set_kv_splits and friends); 0 = automatic.
struct PlanKnobs {
    int32_t forced_splits = 0;
    int32_t forced_row_blocks = 0;
    int32_t forced_attn_kernel = 0;   // 1 general, 2 pipelined, 3 decode (where it applies), 4 long launches
};

// Attention work list for the batch in `p` (host arrays filled in).  Items of one
// (query, KV head, split) read the same K/V; they are given work-group ids that are congruent
// modulo 8 so that they land on the same XCD and share its L2 (work-groups go to the 8 XCDs
// round-robin by id).  Holes are padded with no-op items (q = -1).
// `pipe_cap` is the number of key tiles whose block ids one work item of the kernel in question may
// keep in LDS; returns false if an item came out longer than its kernel allows (a bug: the caller
// refuses the batch rather than launch it).
inline bool plan_attention_pass(const tc_config &c, const PlanKnobs &knobs, Plan &p, std::vector<AttnItem> &items,
                                std::vector<int32_t> &splits_of_q, std::vector<MergeGroup> &groups,
                                int general_cap, bool &cap_bound)
{
    const PlanKnobs *ctx = &knobs;
    cap_bound = false;
    items.clear();                                      // a second pass starts from nothing
    groups.clear();
    const int G = c.n_q_heads / c.n_kv_heads;
    const bool bf16 = c.dtype == TC_BF16;
    const int KT = bf16 ? kAttnKeys : kF32Keys;
    p.decode = false;
    p.pingpong = false;
    // Decode step: every query brings at most one new token, so a KV head has only G rows and the
    // work is reading K and V once.  The decode kernels split the keys of a (query, KV head) over
    // the four waves of a work-group and over `ns` work-groups.  A work-group holds a CU (its ring of
    // tiles fills the LDS), and what a launch of this kind costs is how its loads get going and
    // drain, once per round of work-groups: so the ranges are cut for ONE round of equally long
    // work-groups - the smallest range length L (in key tiles, at least six) for which
    // sum over (query, KV head) of ceil(tiles / L) fits the 256 CUs; a long sequence is cut into
    // more ranges than a short one.  Batches that do not fit one round even at the longest range a
    // work item may have run in several, longest items first.  Unused block tails of sequences that
    // alias table slots ride in the device block table and are masked by the kernel.
    if (bf16 && G <= 32 && p.total_S > 0 && ctx->forced_row_blocks == 0 &&
        (ctx->forced_attn_kernel == 0 || ctx->forced_attn_kernel == 3) &&
        std::all_of(p.suffix_len.begin(), p.suffix_len.end(), [](int32_t s) { return s <= 1; })) {
        constexpr int kCus = 256, kMinRange = 6;
        auto tiles_of_q = [&](int i) { return (p.prefix_len[i] + KT - 1) / KT; };
        auto items_at = [&](int L) {
            int64_t n = 0;
            for (int i = 0; i < p.B; ++i)
                if (p.suffix_len[i] > 0) n += (int64_t)c.n_kv_heads * std::max(1, (tiles_of_q(i) + L - 1) / L);
            return n;
        };
        int L = kAttnMaxTiles;
        if (items_at(L) <= kCus) {                      // one round is possible: the shortest ranges that still fit it
            int lo = kMinRange, hi = kAttnMaxTiles;     // items_at is non-increasing in L
            while (lo < hi) {
                const int mid = (lo + hi) / 2;
                if (items_at(mid) <= kCus) hi = mid;
                else lo = mid + 1;
            }
            L = lo;
        }
        splits_of_q.assign(p.B, 1);
        p.max_splits = 1;
        items.clear();
        groups.clear();
        for (int i = 0; i < p.B; ++i) {
            if (p.suffix_len[i] <= 0) continue;
            const int P = p.prefix_len[i];
            const int n_tiles = tiles_of_q(i);
            int ns = ctx->forced_splits > 0 ? ctx->forced_splits : (n_tiles + L - 1) / L;
            ns = std::max(ns, (n_tiles + kAttnMaxTiles - 1) / kAttnMaxTiles);
            ns = std::max(1, std::min(ns, std::max(n_tiles, 1)));
            splits_of_q[i] = ns;
            p.max_splits = std::max(p.max_splits, ns);
            const int32_t *bt = p.block_table.data() + (size_t)i * p.max_blocks;
            for (int h = 0; h < c.n_kv_heads; ++h)
                for (int s = 0; s < ns; ++s) {
                    AttnItem it{};
                    it.q = i; it.kvh = h; it.tile_begin = (int32_t)((int64_t)n_tiles * s / ns);
                    it.tile_end = (int32_t)((int64_t)n_tiles * (s + 1) / ns);
                    it.split = s; it.n_splits = ns; it.P = P; it.S = 1; it.cu = p.cu_seqlens[i];
                    for (int k = 0; k < 16; ++k) it.bid[k] = bt[0];
                    items.push_back(it);
                }
        }
        std::stable_sort(items.begin(), items.end(), [](const AttnItem &x, const AttnItem &y) {
            return x.tile_end - x.tile_begin > y.tile_end - y.tile_begin;
        });
        p.n_groups = 0;
        p.row_blocks = 1;
        p.n_items = (int32_t)items.size();
        p.pipelined = false;
        p.decode = true;
        for (const AttnItem &it : items)
            if (it.tile_end - it.tile_begin > kAttnMaxTiles) return false;
        return true;
    }
    // key tiles of a query.  bf16 kernel: the tiles of the prefix (from the pool), then the tiles of
    // the suffix (from k_new / v_new); fp32 kernel: one paged sequence of P + S keys
    // the alternating-groups bf16 kernel reads the suffix from the pool as well (it is appended by a
    // launch of its own first), so it, too, sees one paged sequence
    // It is chosen for long launches (estimated from the row tiles x key tiles of the batch at
    // ~0.85 us per 128 x 64 tile and CU): its own append launch costs ~10 us, and with 256 rows per
    // work-group a short launch would not fill the chip.  Measured: c3 (1140 items of ~24 tiles)
    // 207 + 12 us against 226 us in the general kernel, c4 775 + 14 us against 814 us in the pipelined
    // one; c2 (17 us) and the micro-batches of the loading pipeline stay with the other kernels.
    bool pp = false;
    if (bf16 && ctx->forced_row_blocks == 0) {
        if (ctx->forced_attn_kernel == 4) pp = true;
        else if (ctx->forced_attn_kernel == 0) {
            double work = 0;
            for (int i = 0; i < p.B; ++i)
                if (p.suffix_len[i] > 0)
                    work += (double)c.n_kv_heads * ((p.suffix_len[i] * G + kAttnRows - 1) / kAttnRows) *
                            ((p.prefix_len[i] + p.suffix_len[i] + KT - 1) / KT);
            pp = work * 0.85 / 256.0 >= 80.0;
        }
    }
    const bool unified = !bf16 || pp;
    p.pingpong = pp;
    auto tiles_of = [&](int P, int S) {
        return unified ? (P + S + KT - 1) / KT : (P + KT - 1) / KT + (S + KT - 1) / KT;
    };
    // bf16: 128 rows per work-group; 256 (two row blocks per wave, half the LDS traffic per flop but one
    // wave per SIMD) is kept as an option: it is slower until its matrix and vector work overlap
    const int rb = pp ? 2 : (bf16 && ctx->forced_row_blocks > 0) ? ctx->forced_row_blocks : 1;
    p.row_blocks = rb;
    const int RT = bf16 ? kAttnRows * rb : kF32Rows;
    int64_t base = 0, tiles_sum = 0, n_q = 0;
    for (int i = 0; i < p.B; ++i)
        if (p.suffix_len[i] > 0) {
            base += (int64_t)c.n_kv_heads * ((p.suffix_len[i] * G + RT - 1) / RT);
            tiles_sum += tiles_of(p.prefix_len[i], p.suffix_len[i]);
            ++n_q;
        }
    // Number of key partitions: a small cost model, in units of one key tile of one work-group
    // (~1.4 us).  The work items of one (query, KV head, partition) - a bucket - go to one XCD (they
    // share its L2), so what counts is the most loaded XCD: buckets per XCD x items per bucket over
    // its 32 CUs gives the work-groups per CU (a whole number while the chip is not full: 35 items
    // on an XCD mean 3 CUs run two and the launch takes as long as with 64); times the key tiles per
    // work-group (co-resident work-groups overlap each other's stalls: x0.7); plus a fixed start-up
    // and epilogue cost; plus the merge: a launch and the partials written and read back at about
    // 4 TB/s.  Fitted to split-count sweeps and per-work-group traces on c2, c3 and c5-sized batches.
    int want = 1;
    if (ctx->forced_splits > 0) want = ctx->forced_splits;
    else if (base > 0) {
        const double tiles = (double)tiles_sum / (double)n_q;
        const double items_per_bucket = (double)base / (double)(n_q * c.n_kv_heads);
        const double rows = (double)p.total_S * c.n_q_heads;
        double best = 1e30;
        for (int ns = 1; ns <= 32; ++ns) {
            if (ns > 1 && tiles / ns < 2.0) break;
            const double load = std::ceil((double)n_q * c.n_kv_heads * ns / 8.0) * items_per_bucket / 32.0;
            const double per_cu = load <= 1.0 ? 1.0 : (load <= 2.0 ? 2.0 : load);
            const double merge = ns > 1 ? 1.0 + 0.93e-4 * ns * rows : 0.0;   // fp16 partials: 264 B per row and partition
            // (two work-groups on a CU overlap each other's stalls; the long-launch kernel runs one per CU)
            const double cost = per_cu * (tiles / ns) * (per_cu >= 2.0 && !pp ? 0.7 : 1.0) + 3.0 + merge;
            if (cost < best - 1e-9) { best = cost; want = ns; }
        }
    }
    splits_of_q.assign(p.B, 1);
    p.max_splits = 1;
    std::vector<std::vector<AttnItem>> buckets;     // items of one (query, KV head, partition)
    int n_groups = 0;
    for (int i = 0; i < p.B; ++i) {
        const int S = p.suffix_len[i], P = p.prefix_len[i];
        if (S <= 0) continue;
        const int n_tiles = tiles_of(P, S);
        // last block a tile load may touch: bf16 reads only prefix blocks from the pool
        const int last_blk = std::max(0, (unified ? (P + S + kBlockTokens - 1) / kBlockTokens
                                                  : (P + kBlockTokens - 1) / kBlockTokens) - 1);
        int ns = std::min(want, ctx->forced_splits > 0 ? n_tiles : std::max(1, n_tiles / 2));
        const int cap = !bf16 ? n_tiles : pp ? kPpMaxTiles : general_cap;   // block ids of a range fit LDS
        if (ns < (n_tiles + cap - 1) / cap) { ns = (n_tiles + cap - 1) / cap; cap_bound = true; }
        ns = std::max(1, std::min(ns, n_tiles));
        const int n_mt = (S * G + RT - 1) / RT;
        // Partition boundaries.  A suffix tile of the bf16 kernel costs about 4 prefix tiles (its V
        // is transposed on the way into LDS), so the tiles are cut by weight, not by count - and a
        // cut by weight can leave a partition of prefix tiles longer than n_tiles / ns: where one
        // comes out longer than the block-id table allows, the query is cut into more.
        std::vector<int> cut;
        for (;; ++ns) {
            cut.assign(ns + 1, 0);
            const int npt = unified ? n_tiles : (P + KT - 1) / KT;
            const int w_new = 4;
            const int64_t total_w = npt + (int64_t)(n_tiles - npt) * w_new;
            int t = 0;
            int64_t acc = 0;
            for (int s = 1; s < ns; ++s) {
                const int64_t goal = total_w * s / ns;
                while (t < n_tiles - (ns - s) && acc + (t < npt ? 1 : w_new) <= goal) { acc += (t < npt ? 1 : w_new); ++t; }
                if (t < s) { acc += (t < npt ? 1 : w_new); ++t; }        // every partition gets a tile
                cut[s] = t;
            }
            cut[ns] = n_tiles;
            int longest = 0;
            for (int s = 0; s < ns; ++s) longest = std::max(longest, cut[s + 1] - cut[s]);
            if (longest <= cap || ns >= n_tiles) break;
            cap_bound = true;
        }
        splits_of_q[i] = ns;
        p.max_splits = std::max(p.max_splits, ns);
        const int32_t *bt = p.block_table.data() + (size_t)i * p.max_blocks;
        const uint8_t *pad_of = p.block_pad.empty() ? nullptr : p.block_pad.data() + (size_t)i * p.max_blocks;
        for (int h = 0; h < c.n_kv_heads; ++h) {
            for (int s = 0; s < ns; ++s) {
                const int t0 = cut[s], t1 = cut[s + 1];
                std::vector<AttnItem> bucket;
                for (int mt = 0; mt < n_mt; ++mt) {
                    AttnItem it{};
                    it.q = i; it.kvh = h; it.m0 = mt * RT; it.tile_begin = t0; it.tile_end = t1;
                    it.split = s; it.n_splits = ns; it.group = n_groups + mt;
                    it.P = P; it.S = S; it.cu = p.cu_seqlens[i];
                    for (int k = 0; k < 16; ++k) {
                        const int idx = std::min(t0 * (KT / kBlockTokens) + k, last_blk);
                        it.bid[k] = bt[idx] | (pad_of ? (int32_t)((uint32_t)pad_of[idx] << kPadShift) : 0);
                    }
                    if (pad_of && bf16 && !pp) {
                        const int n_fast = std::min(t1, P >> 6) - t0;
                        for (int k = t0 * 4; k < (t0 + std::max(n_fast, 0)) * 4; ++k) it.n_pad_fast += pad_of[k];
                    }
                    bucket.push_back(it);
                }
                buckets.push_back(std::move(bucket));
            }
            for (int mt = 0; mt < n_mt; ++mt) groups.push_back(MergeGroup{h, mt * RT, ns, p.cu_seqlens[i], S, {0, 0, 0}});
            n_groups += n_mt;
        }
    }
    p.n_groups = n_groups;
    // Longest buckets first, each to the XCD with the least work so far (key tiles x items): long
    // work-groups start early, XCDs finish together.
    std::stable_sort(buckets.begin(), buckets.end(), [](const std::vector<AttnItem> &x, const std::vector<AttnItem> &y) {
        return x[0].tile_end - x[0].tile_begin > y[0].tile_end - y[0].tile_begin;
    });
    std::vector<std::vector<AttnItem>> per_xcd(8);
    int64_t xcd_load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (auto &bk : buckets) {
        int xcd = 0;
        for (int x = 1; x < 8; ++x)
            if (xcd_load[x] < xcd_load[xcd]) xcd = x;
        xcd_load[xcd] += (int64_t)(bk[0].tile_end - bk[0].tile_begin + 3) * (int64_t)bk.size();
        for (auto &it : bk) { it.n_groups = n_groups; per_xcd[xcd].push_back(it); }
    }
    size_t longest = 0;
    for (auto &v : per_xcd) longest = std::max(longest, v.size());
    items.clear();
    for (size_t k = 0; k < longest; ++k)
        for (int x = 0; x < 8; ++x)
            if (k < per_xcd[x].size()) items.push_back(per_xcd[x][k]);
            else { AttnItem pad{}; pad.q = -1; pad.n_splits = 1; items.push_back(pad); }
    while (!items.empty() && items.back().q < 0) items.pop_back();
    p.n_items = (int32_t)items.size();
    // Which bf16 kernel (one row block per wave).  The pipelined one holds 132 KB of LDS, so one
    // work-group per CU: nothing hides a work-group's start-up and drain.  It wins when a launch is a
    // single round of work-groups or when they are long; many short ones (measured: 1140 work-groups
    // of ~20 key tiles, 743 vs 647 TFLOP/s) are better off two per CU in the general kernel.
    int64_t n_real = 0, fast_tiles = 0;
    for (const AttnItem &it : items)
        if (it.q >= 0) {
            ++n_real;
            fast_tiles += std::max(std::min(it.tile_end, it.P >> 6) - it.tile_begin, 0);
        }
    p.pipelined = bf16 && rb == 1 && !pp && n_real > 0 &&
                  (ctx->forced_attn_kernel == 1 || ctx->forced_attn_kernel == 2 ? ctx->forced_attn_kernel == 2
                                           : (n_real <= 2 * 256 || fast_tiles >= 48 * n_real));
    // every range's block ids must fit the table of the kernel that will run it
    const int limit = !bf16 ? INT32_MAX : pp ? kPpMaxTiles : p.pipelined ? kPipeMaxTiles : kAttnMaxTiles;
    for (const AttnItem &it : items)
        if (it.q >= 0 && it.tile_end - it.tile_begin > limit) return false;
    return true;
}

// Attention work list of the batch in `p`.  The general kernel keeps the block ids of at most
// kAttnMaxTiles key tiles per work item in LDS, the pipelined kernel (one work-group per CU, LDS to
// spare) kPipeMaxTiles: the batch is planned for the smaller table first; if that limit forced extra
// partitions and the pipelined kernel is the one chosen, it is planned again for the larger one
// (c4's 393-tile queries then run unsplit: no partials, no merge launch).
inline bool plan_attention(const tc_config &c, const PlanKnobs &knobs, Plan &p, std::vector<AttnItem> &items,
                           std::vector<int32_t> &splits_of_q, std::vector<MergeGroup> &groups)
{
    bool cap_bound = false;
    if (!plan_attention_pass(c, knobs, p, items, splits_of_q, groups, kAttnMaxTiles, cap_bound)) return false;
    if (cap_bound && p.pipelined && !p.pingpong && !p.decode) {
        PlanKnobs k2 = knobs;
        k2.forced_attn_kernel = 2;
        if (!plan_attention_pass(c, k2, p, items, splits_of_q, groups, kPipeMaxTiles, cap_bound)) return false;
    }
    return true;
}



}  // namespace tc
