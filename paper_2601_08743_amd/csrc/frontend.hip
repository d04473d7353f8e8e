// Host-side front end, upstream of the hot path (pure C++, no device code): the Table Trie with
// the matching loop of Alg. 1 (paper Sec. 4.1.2) and the greedy query reranking of Sec. 4.2.1
// (Eq. 1-2).  It turns a prompt's token ids into the table_ids that tc_stitch_kv takes, and a
// batch's table sets into a cache-friendly visiting order.
#include "../../include/tablecache.h"

#include <cstdint>
#include <cstring>
#include <new>
#include <unordered_map>
#include <vector>

// Trie over token ids.  Nodes are numbered; edges live in one hash map keyed by (node, token); a
// node that ends a table's content stores that table's id (Sec. 4.1.2: the leaves hold the table id
// and where its KV is - here the id is what tc_register_table_kv knows the KV by).
struct tc_trie {
    std::unordered_map<uint64_t, int32_t> edge;
    std::vector<int32_t> table_of_node{-1};       // node 0 = root
    std::vector<int32_t> ids;                     // inserted table ids (to refuse duplicates)
    static uint64_t key(int32_t node, int32_t tok) { return ((uint64_t)(uint32_t)node << 32) | (uint32_t)tok; }
};

extern "C" {

tc_trie *tc_trie_create(void) { return new (std::nothrow) tc_trie(); }

void tc_trie_destroy(tc_trie *t) { delete t; }

tc_status tc_trie_insert(tc_trie *t, int32_t table_id, const int32_t *tokens, int32_t n_tokens)
{
    if (!t || table_id < 0 || !tokens || n_tokens <= 0) return TC_ERR_INVALID;
    for (int32_t id : t->ids)
        if (id == table_id) return TC_ERR_INVALID;
    // walk first without modifying: a table whose content is already a table's content is refused
    int32_t node = 0;
    int32_t k = 0;
    for (; k < n_tokens; ++k) {
        auto it = t->edge.find(tc_trie::key(node, tokens[k]));
        if (it == t->edge.end()) break;
        node = it->second;
    }
    if (k == n_tokens && t->table_of_node[node] >= 0) return TC_ERR_INVALID;
    try {
        for (; k < n_tokens; ++k) {
            const int32_t next = (int32_t)t->table_of_node.size();
            t->table_of_node.push_back(-1);
            t->edge.emplace(tc_trie::key(node, tokens[k]), next);
            node = next;
        }
        t->ids.push_back(table_id);
    } catch (...) {
        return TC_ERR_INVALID;
    }
    t->table_of_node[node] = table_id;
    return TC_OK;
}

// Alg. 1.  p = 0; at p walk the trie along s[p..] remembering the deepest node that ends a table
// (the longest table that is a prefix of the rest of the prompt); found -> emit it and jump behind
// it, else p + 1.
int32_t tc_trie_match(const tc_trie *t, const int32_t *s, int32_t len, int32_t *table_ids_out,
                      int32_t *start_out, int32_t cap)
{
    if (!t || len < 0 || cap < 0 || (len > 0 && !s) || (cap > 0 && !table_ids_out)) return TC_ERR_INVALID;
    int32_t n = 0, p = 0;
    while (p < len) {
        int32_t node = 0, best_id = -1, best_end = p;
        for (int32_t k = p; k < len; ++k) {
            auto it = t->edge.find(tc_trie::key(node, s[k]));
            if (it == t->edge.end()) break;
            node = it->second;
            if (t->table_of_node[node] >= 0) { best_id = t->table_of_node[node]; best_end = k + 1; }
        }
        if (best_id < 0) { ++p; continue; }
        if (n < cap) {
            table_ids_out[n] = best_id;
            if (start_out) start_out[n] = p;
        }
        ++n;
        p = best_end;
    }
    return n;
}

// Sec. 4.2.1.  I_i = bitset of query i's tables (Eq. 1), d_ij = popcount(I_i xor I_j) (Eq. 2);
// from the anchor, always go to the remaining query nearest to the current one (lowest index on
// ties).  O(N^2 n / 64).
tc_status tc_rerank(const int32_t *table_ids, const int32_t *cu_tables, int32_t n_queries, int32_t n_tables,
                    int32_t anchor, int32_t *order_out)
{
    if (n_queries < 0 || n_tables < 0) return TC_ERR_INVALID;
    if (n_queries == 0) return TC_OK;
    if (!cu_tables || !order_out || anchor < 0 || anchor >= n_queries || cu_tables[0] != 0) return TC_ERR_INVALID;
    const size_t words = ((size_t)n_tables + 63) / 64;
    std::vector<uint64_t> bits;
    std::vector<char> used;
    try {
        bits.assign((size_t)n_queries * (words ? words : 1), 0);
        used.assign(n_queries, 0);
    } catch (...) {
        return TC_ERR_INVALID;
    }
    const size_t stride = words ? words : 1;
    for (int32_t i = 0; i < n_queries; ++i) {
        if (cu_tables[i + 1] < cu_tables[i]) return TC_ERR_INVALID;
        for (int32_t k = cu_tables[i]; k < cu_tables[i + 1]; ++k) {
            if (!table_ids) return TC_ERR_INVALID;
            const int32_t id = table_ids[k];
            if (id < 0 || id >= n_tables) return TC_ERR_INVALID;
            bits[i * stride + (size_t)id / 64] |= 1ull << (id % 64);
        }
    }
    int32_t cur = anchor;
    used[cur] = 1;
    order_out[0] = cur;
    for (int32_t step = 1; step < n_queries; ++step) {
        int32_t best = -1;
        int64_t best_d = INT64_MAX;
        const uint64_t *a = &bits[cur * stride];
        for (int32_t j = 0; j < n_queries; ++j) {
            if (used[j]) continue;
            const uint64_t *b = &bits[j * stride];
            int64_t d = 0;
            for (size_t w = 0; w < words; ++w) d += __builtin_popcountll(a[w] ^ b[w]);
            if (d < best_d) { best_d = d; best = j; }
        }
        used[best] = 1;
        order_out[step] = best;
        cur = best;
    }
    return TC_OK;
}

// Sec. 4.2.2.  The window of requests whose tables are on the device (or on their way) but
// whose stitch has not been issued slides over the ordered batch; `held` counts, per table, the
// window's requests that use it, so its size is the number of slots the window pins.
int32_t tc_plan_pipeline(const int32_t *table_ids, const int32_t *cu_tables, int32_t n_queries,
                         int32_t capacity, int32_t b_c, int32_t b_m, int32_t keep_pinned, int32_t taper,
                         tc_pipe_step *steps_out, int32_t cap)
{
    if (n_queries < 0 || capacity < 0 || b_c < 1 || b_m < 0 || cap < 0) return TC_ERR_INVALID;
    if (n_queries == 0) return 0;
    if (!cu_tables || cu_tables[0] != 0) return TC_ERR_INVALID;
    for (int32_t i = 0; i < n_queries; ++i)
        if (cu_tables[i + 1] < cu_tables[i]) return TC_ERR_INVALID;
    if (cu_tables[n_queries] > 0 && !table_ids) return TC_ERR_INVALID;
    if (!steps_out && cap > 0) return TC_ERR_INVALID;

    std::unordered_map<int32_t, int32_t> held;
    auto add = [&](int32_t i) { for (int32_t k = cu_tables[i]; k < cu_tables[i + 1]; ++k) ++held[table_ids[k]]; };
    auto drop = [&](int32_t i) {
        for (int32_t k = cu_tables[i]; k < cu_tables[i + 1]; ++k) {
            auto it = held.find(table_ids[k]);
            if (--it->second == 0) held.erase(it);
        }
    };
    auto fresh = [&](int32_t i) {      // tables of request i the window does not hold yet
        int32_t n = 0;
        for (int32_t k = cu_tables[i]; k < cu_tables[i + 1]; ++k) {
            bool seen = held.count(table_ids[k]) != 0;
            for (int32_t j = cu_tables[i]; j < k && !seen; ++j) seen = table_ids[j] == table_ids[k];
            n += seen ? 0 : 1;
        }
        return n;
    };

    int32_t frontier = 0;              // requests [0, frontier) have been asked for
    int32_t n_steps = 0;
    for (int32_t c0 = 0; c0 < n_queries; ++n_steps) {
        if (n_steps >= cap) return TC_ERR_INVALID;
        tc_pipe_step &st = steps_out[n_steps];
        // with `taper` the last micro-batches halve (.., b_c, b_c/2, .., 2, 1, 1): what is computed
        // after the final copy has landed is one request instead of b_c
        int32_t size = b_c;
        if (taper) {
            const int32_t half = (n_queries - c0) / 2;
            size = half < 1 ? 1 : (half < b_c ? half : b_c);
        }
        const int64_t full = (int64_t)c0 + size < n_queries ? c0 + size : n_queries;
        st.compute_begin = c0;
        st.demand_begin = frontier;
        // the step takes what has been asked for already (at most b_c requests) and asks for more
        // of its b_c requests while their tables still fit beside the ones held
        while (frontier < full && (int64_t)held.size() + fresh(frontier) <= capacity) add(frontier++);
        st.compute_end = frontier < full ? frontier : (int32_t)full;
        if (st.compute_end == c0) return TC_ERR_CAPACITY;       // one request alone outgrows the cache
        st.demand_end = frontier;
        // a copying stitch is done with the tables once it is enqueued; an aliasing one leaves the
        // attention layers reading them, so they stay held while the prefetch is sized
        if (!keep_pinned)
            for (int32_t i = c0; i < st.compute_end; ++i) drop(i);
        st.prefetch_begin = frontier;
        const int64_t want = (int64_t)st.compute_end + b_m;      // (b_m is not tapered: the copies should stay ahead)
        while (frontier < n_queries && frontier < want && (int64_t)held.size() + fresh(frontier) <= capacity)
            add(frontier++);
        st.prefetch_end = frontier;
        if (keep_pinned)
            for (int32_t i = c0; i < st.compute_end; ++i) drop(i);
        c0 = st.compute_end;
    }
    return n_steps;
}

}  // extern "C"
