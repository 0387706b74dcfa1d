// Host-only checks of the library's bookkeeping code, built with the address and undefined-behaviour sanitizers
// (tests/test_host_sanitizers.py compiles and runs this; no GPU is touched):
//   host_checks sched   reads a scheduling trace from stdin, drives pc_sched_* (the real scheduler source),
//                       prints every output; the test compares them with the oracle's
//   host_checks book N  N random prefill / fork / decode / release operations on the KV bookkeeping (the real
//                       kv_book.h) with every invariant checked after each
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <set>
#include <vector>

#include "../../paper_2605_26606_amd/csrc/index_maps.h"
#include "../../paper_2605_26606_amd/csrc/kv_book.h"
#include "../../paper_2605_26606_amd/csrc/scheduler.hip"

namespace pc {
void set_error(const char *, ...) {}
}

#define REQUIRE(cond)                                                         \
    do {                                                                      \
        if (!(cond)) {                                                        \
            fprintf(stderr, "invariant failed: %s (line %d)\n", #cond, __LINE__); \
            exit(1);                                                          \
        }                                                                     \
    } while (0)

static int run_sched() {
    pc_sched_config cfg;
    if (scanf("S %f %f %f %d %d", &cfg.p_lower, &cfg.p_upper, &cfg.p_solve, &cfg.b_t, &cfg.max_delay) != 5) return 2;
    pc_sched *s = nullptr;
    REQUIRE(pc_sched_create(&cfg, &s) == PC_OK);
    char op[8];
    while (scanf("%7s", op) == 1) {
        if (!strcmp(op, "P")) {
            int n;
            REQUIRE(scanf("%d", &n) == 1 && n >= 0);
            std::vector<int64_t> uid(n), tag(n);
            std::vector<float> ph(n);
            for (int i = 0; i < n; ++i) {
                long long u, t;
                REQUIRE(scanf("%lld %lld %f", &u, &t, &ph[i]) == 3);
                uid[i] = u;
                tag[i] = t;
            }
            std::vector<uint8_t> cls(n + 1), ev(n + 1);
            int32_t counts[4];
            REQUIRE(pc_sched_pilot(s, uid.data(), tag.data(), ph.data(), n, cls.data(), ev.data(), counts) == PC_OK);
            printf("P");
            for (int i = 0; i < n; ++i) printf(" %d%d", cls[i], ev[i]);
            printf(" | %d %d %d %d\n", counts[0], counts[1], counts[2], counts[3]);
        } else if (!strcmp(op, "C")) {
            int64_t st[PC_SCHED_NSTATS];
            REQUIRE(pc_sched_stats(s, st) == PC_OK);
            const int cap = (int)st[PC_SCHED_BUFFERED_NOW];
            std::vector<int64_t> uid(cfg.b_t + 1), tag(cfg.b_t + 1), auid(cap + 1), atag(cap + 1);
            std::vector<int32_t> age(cfg.b_t + 1);
            int32_t k = 0, a = 0;
            REQUIRE(pc_sched_commit(s, uid.data(), tag.data(), age.data(), &k, auid.data(), atag.data(), cap, &a) == PC_OK);
            printf("C");
            for (int i = 0; i < k; ++i) printf(" %lld:%lld:%d", (long long)uid[i], (long long)tag[i], age[i]);
            printf(" |");
            for (int i = 0; i < a; ++i) printf(" %lld:%lld", (long long)auid[i], (long long)atag[i]);
            printf("\n");
        } else if (!strcmp(op, "E")) {
            int n;
            REQUIRE(scanf("%d", &n) == 1 && n >= 0);
            std::vector<int64_t> uid(n);
            for (int i = 0; i < n; ++i) {
                long long u;
                REQUIRE(scanf("%lld", &u) == 1);
                uid[i] = u;
            }
            std::vector<uint8_t> out(n + 1);
            REQUIRE(pc_sched_evicted(s, uid.data(), n, out.data()) == PC_OK);
            printf("E");
            for (int i = 0; i < n; ++i) printf(" %d", out[i]);
            printf("\n");
        } else if (!strcmp(op, "T")) {
            int64_t st[PC_SCHED_NSTATS];
            REQUIRE(pc_sched_stats(s, st) == PC_OK);
            printf("T");
            for (int i = 0; i < PC_SCHED_NSTATS; ++i) printf(" %lld", (long long)st[i]);
            printf("\n");
        } else {
            return 2;
        }
    }
    REQUIRE(pc_sched_destroy(s) == PC_OK);
    return 0;
}

static void check_book(const pc::KvBook &b) {
    std::vector<int> refs((size_t)b.n_blocks, 0);
    size_t used = 0;
    for (int s = 0; s < b.max_slots; ++s) {
        const pc::Slot &sl = b.slots[s];
        if (!sl.used) {
            REQUIRE(sl.blocks.empty());
            continue;
        }
        ++used;
        REQUIRE(sl.len >= 1 && sl.len <= sl.limit && sl.limit <= sl.capacity);
        REQUIRE((int)sl.blocks.size() * b.block_size == sl.capacity && (int)sl.blocks.size() <= b.max_blocks_per_slot);
        for (size_t i = 0; i < sl.blocks.size(); ++i) {
            REQUIRE(sl.blocks[i] >= 0 && sl.blocks[i] < b.n_blocks);
            refs[sl.blocks[i]]++;
            REQUIRE(b.h_table[(size_t)s * b.max_blocks_per_slot + i] == sl.blocks[i]);
        }
        REQUIRE(b.h_len[s] == sl.len);
        if (!sl.is_prompt) {   // a sequence shares exactly the full blocks of its live prompt
            REQUIRE(b.live_prompt(sl.prompt));
            const pc::Slot &ps = b.slots[sl.prompt];
            for (int i = 0; i < ps.len / b.block_size; ++i) REQUIRE(sl.blocks[i] == ps.blocks[i]);
            for (size_t i = ps.len / b.block_size; i < sl.blocks.size(); ++i) REQUIRE(b.refcnt[sl.blocks[i]] == 1);
        }
    }
    REQUIRE(used + b.free_slots.size() == (size_t)b.max_slots);
    std::set<int32_t> free_set(b.free_blocks.begin(), b.free_blocks.end());
    REQUIRE(free_set.size() == b.free_blocks.size());
    size_t in_use = 0;
    for (int64_t k = 0; k < b.n_blocks; ++k) {
        REQUIRE(refs[k] == b.refcnt[k] || (refs[k] == 0 && free_set.count((int32_t)k)));
        REQUIRE((refs[k] == 0) == (free_set.count((int32_t)k) == 1));
        in_use += refs[k] > 0;
    }
    REQUIRE(in_use + b.free_blocks.size() == (size_t)b.n_blocks);
}

static int run_book(int n_ops) {
    pc::KvBook b;
    const int bs = 32, max_ctx = 200;
    b.init(bs, 48, max_ctx, 160);
    uint64_t rng = 0x9E3779B97F4A7C15ull;
    auto next = [&]() {
        rng ^= rng << 13;
        rng ^= rng >> 7;
        rng ^= rng << 17;
        return (uint32_t)(rng >> 20);
    };
    std::vector<int> prompts, seqs;
    int forks = 0, releases = 0, refused = 0;
    for (int op = 0; op < n_ops; ++op) {
        const uint32_t r = next() % 100;
        if (r < 15) {   // a prompt
            const int len = 1 + (int)(next() % 150);
            if (!b.free_slots.empty() && (size_t)b.prompt_blocks(len) <= b.free_blocks.size())
                prompts.push_back(b.take_prompt(len));
            else
                ++refused;
        } else if (r < 50 && !prompts.empty()) {   // a group of forks of one prompt
            const int p = prompts[next() % prompts.size()];
            const int g = 1 + (int)(next() % 4), new_tokens = (int)(next() % 60);
            if (b.slots[p].len + new_tokens > max_ctx) continue;
            if ((size_t)g <= b.free_slots.size() && (size_t)(g * b.fork_blocks(p, new_tokens)) <= b.free_blocks.size()) {
                std::vector<int32_t> pairs;
                for (int i = 0; i < g; ++i) seqs.push_back(b.take_fork(p, new_tokens, pairs));
                REQUIRE(pairs.size() == (b.slots[p].len % bs ? 2u * g : 0u));
                forks += g;
            } else {
                ++refused;
            }
        } else if (r < 80 && !seqs.empty()) {   // a decode step on a few sequences that still have room
            for (int k = 0; k < 4; ++k) {
                const int s = seqs[next() % seqs.size()];
                if (b.slots[s].len < b.slots[s].limit) b.advance(s);
            }
        } else if (r < 92 && !seqs.empty()) {   // release a sequence
            const size_t i = next() % seqs.size();
            b.release(seqs[i]);
            seqs.erase(seqs.begin() + (long)i);
            ++releases;
        } else if (!prompts.empty()) {   // release a prompt whose sequences are gone
            const size_t i = next() % prompts.size();
            bool busy = false;
            for (int s : seqs) busy = busy || b.slots[s].prompt == prompts[i];
            if (busy) continue;
            b.release(prompts[i]);
            prompts.erase(prompts.begin() + (long)i);
            ++releases;
        }
        check_book(b);
    }
    for (int s : seqs) b.release(s);
    for (int p : prompts) b.release(p);
    check_book(b);
    REQUIRE(b.free_blocks.size() == (size_t)b.n_blocks && b.free_slots.size() == (size_t)b.max_slots);
    printf("book ok: %d operations, %d forks, %d releases, %d refused for lack of room\n", n_ops, forks, releases, refused);
    return 0;
}

// The index maps of the kernels, checked exhaustively: the fragment-order cache layout is a bijection of a block's
// (token, dim) pairs onto its elements in which every operand fragment is 512 consecutive elements with lane
// (i, g) at element (16 g + i) * 8 holding what the matrix-core kernels expect there; the GEMM's patch order
// visits every tile exactly once, gives every die the same number of tiles, and any 32 consecutive tiles of a die
// touch at most 4 row blocks and 8 column blocks (ragged last column group aside).
static int run_maps() {
    using namespace pc;
    for (int hd : {32, 64, 128, 256})
        for (int bs : {32, 64, 128, 256}) {
            std::vector<int> seen_k((size_t)bs * hd, 0), seen_v((size_t)bs * hd, 0);
            for (int t = 0; t < bs; ++t)
                for (int d = 0; d < hd; ++d) {
                    const int k = kv_k_index_frag(t, d, hd), v = kv_v_index_frag(t, d, hd);
                    REQUIRE(k >= 0 && k < bs * hd && v >= 0 && v < bs * hd);
                    seen_k[k]++;
                    seen_v[v]++;
                }
            for (int x : seen_k) REQUIRE(x == 1);
            for (int x : seen_v) REQUIRE(x == 1);
            // what lane (i, g) finds at its place in each fragment
            for (int tile = 0; tile < bs / 32; ++tile)
                for (int g = 0; g < 4; ++g)
                    for (int i = 0; i < 16; ++i)
                        for (int j = 0; j < 8; ++j) {
                            for (int u = 0; u < 2; ++u)
                                for (int kk = 0; kk < hd / 32; ++kk) {
                                    const int tok = 32 * tile + 8 * (i / 4) + i % 4 + 4 * u, dim = 32 * kk + 8 * g + j;
                                    REQUIRE(kv_k_index_frag(tok, dim, hd) ==
                                            (((tile * 2 + u) * (hd / 32) + kk) << 9) + (16 * g + i) * 8 + j);
                                }
                            for (int nn = 0; nn < hd / 16; ++nn) {
                                const int tok = 32 * tile + 8 * g + j, dim = 16 * nn + i;
                                REQUIRE(kv_v_index_frag(tok, dim, hd) == ((tile * (hd / 16) + nn) << 9) + (16 * g + i) * 8 + j);
                            }
                        }
        }
    int checked = 0;
    for (int mb : {8, 16, 24, 32, 40, 64, 128})
        for (int nb : {1, 3, 6, 7, 8, 9, 12, 16, 70, 594, 1187}) {
            std::vector<int> seen((size_t)mb * nb, 0);
            std::vector<std::vector<std::pair<int, int>>> per_die(8);
            int bm = -1, bn = -1;
            for (int id = 0; id < mb * nb; ++id) {
                REQUIRE(gemm_patch_tile(id, mb, nb, &bm, &bn));
                REQUIRE(bm >= 0 && bm < mb && bn >= 0 && bn < nb);
                seen[(size_t)bm * nb + bn]++;
                per_die[id % 8].push_back({bm, bn});
            }
            REQUIRE(!gemm_patch_tile(mb * nb, mb, nb, &bm, &bn));
            for (int x : seen) REQUIRE(x == 1);
            const int ph = ((mb / 8) % 4 == 0) ? 4 : (((mb / 8) % 2 == 0) ? 2 : 1);
            for (int die = 0; die < 8; ++die) {
                REQUIRE((int)per_die[die].size() == mb / 8 * nb);
                for (auto &t : per_die[die]) REQUIRE(t.first / (mb / 8) == die);   // a die keeps to its row blocks
                // aligned windows of ph * 8 tiles inside full column groups are exactly one patch
                const int full_groups = nb / 8, per_group = mb / 8 * 8;
                for (int w0 = 0; w0 + ph * 8 <= full_groups * per_group; w0 += ph * 8) {
                    std::set<int> rows, cols;
                    for (int k = 0; k < ph * 8; ++k) {
                        rows.insert(per_die[die][w0 + k].first);
                        cols.insert(per_die[die][w0 + k].second);
                    }
                    REQUIRE((int)rows.size() == ph && (int)cols.size() == 8);
                }
            }
            ++checked;
        }
    printf("maps ok: cache layouts for 16 geometries, %d tile grids\n", checked);
    return 0;
}

int main(int argc, char **argv) {
    if (argc > 1 && !strcmp(argv[1], "maps")) return run_maps();
    if (argc > 1 && !strcmp(argv[1], "sched")) return run_sched();
    if (argc > 2 && !strcmp(argv[1], "book")) return run_book(atoi(argv[2]));
    fprintf(stderr, "usage: host_checks sched < trace | host_checks book N | host_checks maps\n");
    return 2;
}
