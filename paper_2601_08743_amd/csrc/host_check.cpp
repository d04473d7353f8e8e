// Command-line driver for the library's host-only logic, for builds with a plain C++ compiler and
// the address / undefined-behaviour sanitizers (tests/test_host_sanitized.py; not part of
// libtablecache.so).  It reads a script from standard input and prints what the library's own code -
// the replacement rules of paper App. A, the sequence-block allocator, the attention planner and the
// front end (Table Trie / Alg. 1, reranking of Eq. 1-2, the Sec. 4.2.2 pipeline schedule) - answers;
// the test compares that with the CPU checker's models and with the planner's invariants.
//
//   rule <policy> <capacity>        start a cache under LRU (0) / FIFO (1) / LFU (2)
//   r <id>                          request          -> "r <id> <hit> <evicted | -1 | refused>"
//   p <id> / u <id>                 pin / unpin (counted)
//   seq <first> <end>               start an allocator over blocks [first, end)
//   t <n>                           take the n lowest free blocks -> "t b0 b1 ..."
//   f <k> b0 .. bk-1                release
//   plan <dtype> <Hq> <Hkv> <D> <splits> <row_blocks> <kernel> <B> then B pairs "P S"
//                                   -> "plan <n_items> <max_splits> <decode> <pingpong> <pipelined> <row_blocks> <ok>"
//                                      one line "i q kvh m0 tile_begin tile_end split n_splits group" per item,
//                                      "groups <entries> <n_groups>" and one line "g kvh m0 n_splits cu S" per merge group
//   trie <n> then n lines "<id> <len> tok..."; match <len> tok... -> "match <n> (id start)..."
//   rerank <n_queries> <n_tables> <anchor> then per query "<k> ids..." -> "rerank order..."
//   pipeline <n_queries> <capacity> <b_c> <b_m> <keep_pinned> <taper> then per query "<k> ids..."
//                                   -> "pipeline <n_steps | status>" and one line of six numbers per step
#include "host_logic.h"
#include "frontend.hip"

#include <cstdio>
#include <iostream>
#include <memory>
#include <string>

using namespace tc;

int main()
{
    std::unique_ptr<Replacement> rule;
    PinMap pins;
    int64_t capacity = 0;
    SeqBlocks seq;
    tc_trie *trie = nullptr;
    std::string cmd;
    while (std::cin >> cmd) {
        if (cmd == "rule") {
            int policy;
            std::cin >> policy >> capacity;
            rule.reset(make_rule(policy));
            pins.clear();
        } else if (cmd == "r") {
            int32_t id;
            std::cin >> id;
            const CacheStep s = cache_request(*rule, pins, capacity, id);
            if (s.refused) std::printf("r %d 0 refused\n", id);
            else std::printf("r %d %d %d\n", id, s.hit ? 1 : 0, s.evicted);
        } else if (cmd == "p") {
            int32_t id;
            std::cin >> id;
            pins[id] += 1;
        } else if (cmd == "u") {
            int32_t id;
            std::cin >> id;
            auto it = pins.find(id);
            if (it != pins.end() && --it->second == 0) pins.erase(it);
        } else if (cmd == "seq") {
            int64_t first, end;
            std::cin >> first >> end;
            seq.reset(first, end);
        } else if (cmd == "t") {
            size_t n;
            std::cin >> n;
            std::printf("t");
            if (n <= seq.n_free())
                for (int32_t b : seq.lowest(n)) { seq.take(b); std::printf(" %d", b); }
            else std::printf(" oom");
            std::printf("\n");
        } else if (cmd == "f") {
            int k;
            std::cin >> k;
            for (int j = 0; j < k; ++j) {
                int32_t b;
                std::cin >> b;
                if (seq.allocated(b)) seq.release(b);
                else std::printf("f bad %d\n", b);
            }
        } else if (cmd == "plan") {
            tc_config c{};
            PlanKnobs knobs;
            int B;
            std::cin >> c.dtype >> c.n_q_heads >> c.n_kv_heads >> c.head_dim >> knobs.forced_splits >>
                knobs.forced_row_blocks >> knobs.forced_attn_kernel >> B;
            c.n_layers = 1; c.block_size = kBlockTokens;
            Plan p;
            p.B = B;
            p.cu_seqlens.assign(B + 1, 0);
            int max_blocks = 1;
            for (int i = 0; i < B; ++i) {
                int P, S;
                std::cin >> P >> S;
                p.prefix_len.push_back(P);
                p.suffix_len.push_back(S);
                p.cu_seqlens[i + 1] = p.cu_seqlens[i] + S;
                max_blocks = std::max(max_blocks, (P + S + kBlockTokens - 1) / kBlockTokens);
            }
            p.max_blocks = max_blocks;
            p.total_S = p.cu_seqlens[B];
            p.block_table.assign((size_t)B * max_blocks, -1);
            int32_t next = 1000;
            for (int i = 0; i < B; ++i)
                for (int j = 0; j < (p.prefix_len[i] + p.suffix_len[i] + kBlockTokens - 1) / kBlockTokens; ++j)
                    p.block_table[(size_t)i * max_blocks + j] = next++;
            std::vector<AttnItem> items;
            std::vector<int32_t> splits;
            std::vector<MergeGroup> groups;
            const bool ok = plan_attention(c, knobs, p, items, splits, groups);
            std::printf("plan %d %d %d %d %d %d %d\n", (int)items.size(), p.max_splits, p.decode ? 1 : 0,
                        p.pingpong ? 1 : 0, p.pipelined ? 1 : 0, p.row_blocks, ok ? 1 : 0);
            for (const AttnItem &it : items)
                std::printf("i %d %d %d %d %d %d %d %d\n", it.q, it.kvh, it.m0, it.tile_begin, it.tile_end, it.split, it.n_splits,
                            it.q < 0 ? -1 : it.group);
            std::printf("groups %d %d\n", (int)groups.size(), p.n_groups);
            for (const MergeGroup &mg : groups) std::printf("g %d %d %d %d %d\n", mg.kvh, mg.m0, mg.n_splits, mg.cu, mg.S);
        } else if (cmd == "trie") {
            int n;
            std::cin >> n;
            if (trie) tc_trie_destroy(trie);
            trie = tc_trie_create();
            for (int k = 0; k < n; ++k) {
                int32_t id;
                int len;
                std::cin >> id >> len;
                std::vector<int32_t> toks(len);
                for (int32_t &x : toks) std::cin >> x;
                const tc_status st = tc_trie_insert(trie, id, toks.data(), len);
                if (st != TC_OK) std::printf("trie refused %d\n", id);
            }
        } else if (cmd == "match") {
            int len;
            std::cin >> len;
            std::vector<int32_t> s(len), ids(len + 1), starts(len + 1);
            for (int32_t &x : s) std::cin >> x;
            const int32_t n = tc_trie_match(trie, s.data(), len, ids.data(), starts.data(), len + 1);
            std::printf("match %d", n);
            for (int k = 0; k < n; ++k) std::printf(" %d %d", ids[k], starts[k]);
            std::printf("\n");
        } else if (cmd == "rerank" || cmd == "pipeline") {
            int n_q, a1, a2, a3 = 0, a4 = 0, a5 = 0;
            std::cin >> n_q >> a1 >> a2;
            if (cmd == "pipeline") std::cin >> a3 >> a4 >> a5;
            std::vector<int32_t> ids, cu(1, 0);
            for (int i = 0; i < n_q; ++i) {
                int k;
                std::cin >> k;
                for (int j = 0; j < k; ++j) {
                    int32_t x;
                    std::cin >> x;
                    ids.push_back(x);
                }
                cu.push_back((int32_t)ids.size());
            }
            if (cmd == "rerank") {
                std::vector<int32_t> order(n_q);
                const tc_status st = tc_rerank(ids.data(), cu.data(), n_q, a1, a2, order.data());
                std::printf("rerank");
                if (st != TC_OK) std::printf(" status %d", st);
                else for (int32_t o : order) std::printf(" %d", o);
                std::printf("\n");
            } else {
                std::vector<tc_pipe_step> steps(n_q + 1);
                const int32_t n = tc_plan_pipeline(ids.data(), cu.data(), n_q, a1, a2, a3, a4, a5, steps.data(), n_q + 1);
                std::printf("pipeline %d\n", n);
                for (int k = 0; k < n; ++k)
                    std::printf("s %d %d %d %d %d %d\n", steps[k].compute_begin, steps[k].compute_end, steps[k].demand_begin,
                                steps[k].demand_end, steps[k].prefetch_begin, steps[k].prefetch_end);
            }
        } else {
            std::fprintf(stderr, "host_check: unknown command '%s'\n", cmd.c_str());
            return 2;
        }
    }
    if (trie) tc_trie_destroy(trie);
    return 0;
}
