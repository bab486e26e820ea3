// Random operation sequences on accounting-only caches (no arena, no GPU) and random instances of the allocation
// solver: the program tests/test_host_sanitizers.py builds together with the library's host code under
// AddressSanitizer and UndefinedBehaviorSanitizer.  Argument: number of seeds.  Exit code 0 and no sanitizer report
// = pass; the status codes the calls return are counted, not judged (invalid arguments are part of the mix).
#include "kvq.h"
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include <algorithm>
int main(int argc, char** argv) {
    int seeds = argc > 1 ? atoi(argv[1]) : 200;
    long ops = 0, errs[8] = {0};
    for (int seed = 0; seed < seeds; ++seed) {
        std::mt19937 rng(seed);
        auto R = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
        kvq_config_t cfg{};
        cfg.n_layers = R(1, 3); cfg.batch = R(1, 3); cfg.n_kv_heads = R(1, 4); cfg.n_q_heads = cfg.n_kv_heads * R(1, 8);
        cfg.head_dim = 128; cfg.group = 32 << R(0, 2);
        cfg.page_tokens = 32 * R(1, 4);
        cfg.max_tokens = cfg.page_tokens * R(4, 40);
        cfg.window = cfg.page_tokens * R(0, 2); cfg.n_sink = cfg.page_tokens * R(0, 1);
        cfg.policy = R(0, 1); cfg.count_metadata_in_budget = R(0, 1);
        std::vector<uint64_t> budget((size_t)cfg.n_layers);
        std::vector<uint8_t> fbit((size_t)cfg.n_layers);
        for (int l = 0; l < cfg.n_layers; ++l) {
            fbit[(size_t)l] = (uint8_t)(2 << R(0, 2));
            budget[(size_t)l] = (uint64_t)cfg.batch * cfg.n_kv_heads * (uint64_t)R(cfg.page_tokens * 2, cfg.max_tokens) * (uint64_t)R(96, 520);
        }
        kvq_cache_t* c = nullptr;
        const uint64_t ab = kvq_arena_bytes(&cfg, (uint64_t)cfg.n_layers * cfg.batch * cfg.n_kv_heads * (uint64_t)cfg.max_tokens * 600 * (R(0, 3) ? 1 : 0) + (1 << 20) * (uint64_t)R(0, 4));
        kvq_status_t st = kvq_cache_create(&cfg, budget.data(), fbit.data(), nullptr, ab, &c);
        if (st != KVQ_OK) { errs[st]++; continue; }
        int int16 = 0;
        if (R(0, 3) == 0 && kvq_cache_set_option(c, KVQ_OPT_TIER16, 1) == KVQ_OK) int16 = 1;
        // invariants of the accounting (Sec. 3.1-3.2), checked after every call: the runs of equal width tile
        // [0, T) in order, widths are 16/8/4/2 and not below the block's Fbit (unless the caller itself put tokens
        // at a lower width, which explicit entry widths and the lowering of a named run allow), the bytes in use are the runs' tokens times the bytes
        // of a token at the run's width, and they never exceed the block's budget
        std::vector<char> below((size_t)cfg.n_layers, 0);
        auto check = [&](int when) -> bool {
            for (int l = 0; l < cfg.n_layers; ++l) {
                kvq_segment_info_t segs[256]; int n = 0; uint64_t used = 0; int T = 0, cur = 0;
                if (kvq_cache_describe(c, l, segs, 256, &n, &used, &T, &cur) != KVQ_OK) continue;  // poisoned or > 256 runs
                uint64_t want = 0; int t = 0;
                for (int i = 0; i < n; ++i) {
                    const int b = segs[i].bits;
                    if (segs[i].token_begin != t || segs[i].token_end <= t || (b != 16 && b != 8 && b != 4 && b != 2) ||
                        (b < fbit[(size_t)l] && !below[(size_t)l])) {
                        printf("seed %d op %d: bad run %d of block %d: tokens [%d, %d) at %d bits, previous run ended at %d, Fbit %d\n",
                               seed, when, i, l, segs[i].token_begin, segs[i].token_end, b, t, (int)fbit[(size_t)l]);
                        return false;
                    }
                    want += (uint64_t)(segs[i].token_end - t) * cfg.batch * cfg.n_kv_heads *
                            kvq_bytes_per_token_head(b, 128, cfg.group, cfg.count_metadata_in_budget, int16);
                    t = segs[i].token_end;
                }
                if (t != T || T > cfg.max_tokens || used != want || used > budget[(size_t)l]) {
                    printf("seed %d op %d block %d: T %d/%d, bytes %llu, runs give %llu, budget %llu\n", seed, when, l, t, T,
                           (unsigned long long)used, (unsigned long long)want, (unsigned long long)budget[(size_t)l]);
                    return false;
                }
            }
            return true;
        };
        for (int op = 0; op < 400; ++op, ++ops) {
            if (!check(op)) return 1;
            int layer = R(0, 30) ? R(0, cfg.n_layers - 1) : R(-1, cfg.n_layers);  // sometimes invalid
            int what = R(0, 9);
            if (what <= 5) {
                int n = R(0, 12) ? R(1, 70) : R(-2, cfg.max_tokens + 5);
                int eb = R(0, 4) ? 0 : (R(0, 5) == 5 ? 3 : 2 << R(0, 3));
                st = kvq_quantize_append(c, layer, nullptr, nullptr, n, eb, nullptr);
                errs[st]++;
                if (st == KVQ_OK && eb != 0 && layer >= 0 && layer < cfg.n_layers && eb < fbit[(size_t)layer]) below[(size_t)layer] = 1;
                if (st == KVQ_E_BUDGET) {
                    int done = -1;
                    st = kvq_progressive_requant(c, layer, -1, n > 0 ? n : 0, nullptr, &done);
                    errs[st]++;
                }
            } else if (what == 6) {
                kvq_segment_info_t segs[64]; int n = 0; uint64_t used = 0; int T = 0, cur = 0;
                st = kvq_cache_describe(c, layer, segs, R(0, 64), &n, &used, &T, &cur);
                errs[st]++;
            } else if (what == 7) {
                int done = -1;
                const int seg = R(-1, 6);
                st = kvq_progressive_requant(c, layer, seg, R(0, 40), nullptr, &done);
                errs[st]++;
                // lowering a named run is the policy-free mechanism: it may go below Fbit, like an explicit entry width
                if (st == KVQ_OK && seg >= 0 && layer >= 0 && layer < cfg.n_layers) below[(size_t)layer] = 1;
            } else if (what == 8) {
                if (R(0, 9) == 0) {
                    const int which = R(-1, cfg.n_layers - 1);
                    st = kvq_cache_reset(c, which); errs[st]++;
                    if (st == KVQ_OK) for (int l = 0; l < cfg.n_layers; ++l) if (which < 0 || which == l) below[(size_t)l] = 0;
                }
                else { st = kvq_cache_set_option(c, R(0, 9), R(-1, 300)); errs[st]++; }
            } else {
                float q[4]; st = kvq_decode_attention(c, layer, q, q, 0, 0.f, nullptr); errs[st]++;
                kvq_cache_t* cs[2] = {c, c};
                const void* qs[2] = {q, q}; void* os[2] = {q, q};
                st = kvq_decode_attention_batch(cs, R(0, 2), layer, qs, os, 0, 0.f, nullptr); errs[st]++;
            }
        }
        kvq_cache_destroy(c);
        // allocation solver on random instances (incl. infeasible budgets, zero costs, equal items)
        {
            int nb = R(1, 24), nc = R(1, 4);
            std::vector<double> sv((size_t)(nb * nc));
            std::vector<uint64_t> mv((size_t)(nb * nc));
            uint64_t lo = 0, hi = 0;
            for (int b = 0; b < nb; ++b) {
                uint64_t mn = ~0ull, mx = 0;
                for (int k = 0; k < nc; ++k) {
                    sv[(size_t)(b * nc + k)] = R(0, 5) ? (double)R(0, 100000) / 7.0 : 0.0;
                    mv[(size_t)(b * nc + k)] = (uint64_t)R(0, 9) ? (uint64_t)R(1, 4096) * (R(0, 1) ? 96 : 1) : 0;
                    mn = std::min(mn, mv[(size_t)(b * nc + k)]); mx = std::max(mx, mv[(size_t)(b * nc + k)]);
                }
                lo += mn; hi += mx;
            }
            uint64_t budget_b = R(0, 5) ? lo + (hi - lo) * (uint64_t)R(0, 100) / 100 : (lo ? lo - 1 : 0);
            std::vector<int32_t> choice((size_t)nb);
            double ts = 0; uint64_t tm = 0;
            st = kvq_allocate_bits(nb, nc, sv.data(), mv.data(), budget_b, choice.data(), &ts, &tm);
            errs[st]++;
            if (st == KVQ_OK) {
                uint64_t m = 0;
                for (int b = 0; b < nb; ++b) {
                    if (choice[(size_t)b] < 0 || choice[(size_t)b] >= nc) { printf("bad choice\n"); return 1; }
                    m += mv[(size_t)(b * nc + choice[(size_t)b])];
                }
                if (m != tm || m > budget_b) { printf("allocation over budget: %llu %llu %llu\n", (unsigned long long)m, (unsigned long long)tm, (unsigned long long)budget_b); return 1; }
            }
        }
    }
    printf("ops %ld; status counts:", ops);
    for (int i = 0; i < 8; ++i) printf(" %d:%ld", i, errs[i]);
    printf("\n");
    return 0;
}
