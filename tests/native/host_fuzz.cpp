// CPU-only stress driver for the host side of libspin (tables, decomposition, tiling check,
// scheduler), built with AddressSanitizer and UndefinedBehaviorSanitizer by
// tests/test_host_sanitize.py.  It checks return codes and simple invariants; memory errors and
// undefined behaviour are what the sanitizers are there to catch.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "spin.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main(int argc, char** argv) {
    const int rounds = argc > 1 ? atoi(argv[1]) : 300;
    std::mt19937 rng(12345);
    auto uni = [&](int lo, int hi) { return std::uniform_int_distribution<int>(lo, hi)(rng); };
    for (int round = 0; round < rounds; ++round) {
        const int n_req = uni(0, 12);
        std::vector<int32_t> prefix(n_req), draft(n_req), qoff(n_req + 1, 0);
        for (int i = 0; i < n_req; ++i) {
            prefix[i] = uni(0, 3) == 0 ? uni(0, 20) : uni(0, 6000);
            draft[i] = uni(1, 16);
            qoff[i + 1] = qoff[i] + draft[i];
        }
        spin_req_table t{n_req, prefix.data(), draft.data(), qoff.data(), nullptr, nullptr};

        // decompositions through the library itself, with the capacity protocol
        std::vector<std::vector<spin_subreq>> decomps;
        for (int policy = 0; policy < 4; ++policy) {
            spin_decomp_params p{policy, uni(1, 6), uni(1, 900), uni(1, 4 * (n_req + 1)), uni(1, 64), 6100, uni(1, 32)};
            int32_t n = 0, L = 0;
            int rc = spin_decompose(&t, &p, nullptr, 0, &n, &L);
            if (policy == SPIN_DECOMP_KV_SEARCH && rc == SPIN_ENOSPC && n == 0) continue;   // no L fits: documented
            CHECK(rc == SPIN_OK || rc == SPIN_ENOSPC);
            std::vector<spin_subreq> subs(n);
            rc = spin_decompose(&t, &p, subs.data(), n, &n, &L);
            CHECK(rc == SPIN_OK);
            CHECK(spin_check_tiling(&t, subs.data(), n) == SPIN_OK);
            if (n > 1) {   // one piece short is never a tiling
                CHECK(spin_check_tiling(&t, subs.data() + 1, n - 1) == SPIN_ETABLE);
            }
            decomps.push_back(subs);
        }
        // random 2-D tilings: row bands, each cut along the keys
        {
            std::vector<spin_subreq> subs;
            for (int i = 0; i < n_req; ++i) {
                for (int qb = 0; qb < draft[i];) {
                    const int ql = uni(1, draft[i] - qb);
                    const int end = prefix[i] + qb + ql;
                    for (int kb = 0; kb < end;) {
                        const int kl = uni(1, end - kb);
                        subs.push_back({i, qb, ql, kb, kl});
                        kb += kl;
                    }
                    qb += ql;
                }
            }
            CHECK(spin_check_tiling(&t, subs.data(), (int32_t)subs.size()) == SPIN_OK);
            decomps.push_back(subs);
        }
        // the scheduler on every decomposition, several launch sizes / groups / page sizes
        for (const auto& subs : decomps) {
            const int group = 1 << uni(0, 3), n_kv = uni(1, 5), page = 1 << uni(0, 6), waves = uni(1, 3000);
            int32_t n = 0;
            int rc = spin_schedule(&t, subs.data(), (int32_t)subs.size(), page, group, n_kv, waves, nullptr, 0, &n);
            CHECK(rc == SPIN_OK || rc == SPIN_ENOSPC);
            std::vector<spin_work_piece> pcs(n);
            rc = spin_schedule(&t, subs.data(), (int32_t)subs.size(), page, group, n_kv, waves, pcs.data(), n, &n);
            CHECK(rc == SPIN_OK);
            // per head, the pieces cover exactly the visible cells of every request
            std::vector<int64_t> cells((size_t)n_req * n_kv, 0);
            for (const auto& pc : pcs) {
                CHECK(pc.parent >= 0 && pc.parent < n_req && pc.kv_head >= 0 && pc.kv_head < n_kv);
                CHECK(pc.q_len * group <= 64 && pc.kv_len >= 1);
                for (int r = pc.q_begin; r < pc.q_begin + pc.q_len; ++r) {
                    const int hi = std::min(pc.kv_begin + pc.kv_len, prefix[pc.parent] + r + 1);
                    if (hi > pc.kv_begin) cells[(size_t)pc.parent * n_kv + pc.kv_head] += hi - pc.kv_begin;
                }
            }
            for (int i = 0; i < n_req; ++i)
                for (int h = 0; h < n_kv; ++h) {
                    const int64_t g = draft[i], p = prefix[i];
                    CHECK(cells[(size_t)i * n_kv + h] == g * p + g * (g + 1) / 2);
                }
        }
        // malformed input must be refused, not crash
        if (n_req > 0) {
            std::vector<spin_subreq> bad = decomps.empty() ? std::vector<spin_subreq>() : decomps[0];
            if (!bad.empty()) {
                bad[0].parent = n_req + 3;
                CHECK(spin_check_tiling(&t, bad.data(), (int32_t)bad.size()) == SPIN_ETABLE);
                bad[0].parent = 0;
                bad[0].kv_len = 1 << 30;
                CHECK(spin_check_tiling(&t, bad.data(), (int32_t)bad.size()) == SPIN_ETABLE);
            }
            draft[0] = 0;
            int32_t n = 0;
            spin_decomp_params p{SPIN_DECOMP_NONE, 0, 0, 0, 0, 0, 0};
            CHECK(spin_decompose(&t, &p, nullptr, 0, &n, nullptr) == SPIN_EINVAL);
            draft[0] = 1;
        }
    }
    printf("host fuzz ok: %d rounds\n", rounds);
    return 0;
}
