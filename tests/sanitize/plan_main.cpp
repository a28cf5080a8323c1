// Host-only driver for the sanitizer test: every plan and schedule query of the library's host
// side (plan.cpp) over a list of cluster shapes, all 27 strategy strings, every rank and chunk,
// plus the error paths - built with -fsanitize=address,undefined and run on the CPU.
// Usage: plan_main P:G [P:G ...]
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "plan.hpp"

// the device side (kernels.hip) defines this in the library; here the plan has no device tables
extern "C" void paro_plan_destroy(paro_plan_t *pl) { delete pl; }

static int check(bool ok, const char *what) {
    if (!ok) std::printf("FAILED: %s (%s)\n", what, paro_last_error());
    return ok ? 0 : 1;
}

int main(int argc, char **argv) {
    const char *letters = "NIG";
    long plans = 0, msgs_total = 0, segs_total = 0;
    int bad = 0;
    for (int a = 1; a < argc; ++a) {
        int P = 0, G = 0;
        if (std::sscanf(argv[a], "%d:%d", &P, &G) != 2) return 2;
        for (int x = 0; x < 27; ++x) {
            const char s[4] = {letters[x / 9], letters[(x / 3) % 3], letters[x % 3], 0};
            std::vector<int64_t> sizes = {5, 0, 7, 3, 0, 4099, 1, 20000 + P, 0};
            std::vector<uint8_t> dt = {0, 1, 2, 0, 1, 2, 0, 1, 2}, nd = {0, 1, 0, 1, 0, 1, 0, 1, 1};
            for (int align : {0, 64}) {
                paro_plan_opts_t o = {PARO_SCHED_DEFAULT, align, dt.data(), nd.data(), PARO_BF16, 0};
                paro_plan_t *pl = nullptr;
                const int rc = paro_plan(P, G, s, sizes.data(), (int64_t)sizes.size(), &o, &pl);
                if (!paro_strategy_legal(s)) {
                    bad += check(rc == PARO_ESTRATEGY && pl == nullptr, "an illegal strategy must be refused");
                    continue;
                }
                bad += check(rc == PARO_OK && pl != nullptr, "paro_plan");
                if (rc != PARO_OK) continue;
                ++plans;
                bad += check(paro_padded_total(pl) == (int64_t)P * paro_shard_len(pl), "padded total");
                for (int r = 0; r < P; ++r) {
                    int64_t b, n;
                    for (char st : {'P', 'G', 'O'}) bad += check(paro_range(pl, r, st, &b, &n) == PARO_OK, "paro_range");
                    const int64_t cnt = paro_segments(pl, r, nullptr, 0);
                    bad += check(cnt >= 0, "paro_segments count");
                    std::vector<paro_seg_t> segs((size_t)cnt + 1);
                    bad += check(paro_segments(pl, r, segs.data(), cnt) == cnt, "paro_segments fill");
                    if (cnt > 1) bad += check(paro_segments(pl, r, segs.data(), 1) == cnt, "paro_segments short");
                    segs_total += cnt;
                    int64_t dl, so, sl;
                    bad += check(paro_pack_slot(pl, r, &dl, &so, &sl) == PARO_OK && so + sl <= dl, "paro_pack_slot");
                    bad += check(paro_owner_of_chunk(pl, paro_chunk_of_rank(pl, r)) == r, "owner(chunk(r)) == r");
                    for (int sched : {PARO_SCHED_DEFAULT, PARO_RING, PARO_HRING, PARO_HORING})
                        for (int coll : {PARO_RS, PARO_AG}) {
                            const int64_t m = paro_schedule(pl, r, sched, coll, nullptr, 0);
                            if (m < 0) continue;             // a hierarchical schedule on a cluster without groups
                            std::vector<paro_msg_t> ms((size_t)m + 1);
                            bad += check(paro_schedule(pl, r, sched, coll, ms.data(), m) == m, "paro_schedule fill");
                            for (int64_t k = 0; k < m; ++k)
                                bad += check(ms[(size_t)k].recv_off >= 0 &&
                                                 ms[(size_t)k].recv_off + ms[(size_t)k].recv_len <= paro_padded_total(pl),
                                             "a message stays inside the flat buffer");
                            msgs_total += m;
                        }
                }
                for (int ch = 0; ch < P; ++ch) {
                    std::vector<int32_t> ranks((size_t)P);
                    int32_t gl = 0;
                    bad += check(paro_fold_order(pl, ch, ranks.data(), &gl) == PARO_OK && gl > 0 && P % gl == 0 &&
                                     ranks[(size_t)P - 1] == paro_owner_of_chunk(pl, ch),
                                 "paro_fold_order: the owner adds last");
                }
                // queries out of range must fail cleanly
                int64_t b, n;
                bad += check(paro_range(pl, P, 'O', &b, &n) == PARO_ERANGE && paro_range(pl, -1, 'O', &b, &n) == PARO_ERANGE &&
                                 paro_range(pl, 0, 'X', &b, &n) == PARO_EINVAL && paro_chunk_of_rank(pl, P) < 0 &&
                                 paro_owner_of_chunk(pl, -1) < 0 && paro_segments(pl, P, nullptr, 0) < 0,
                             "out-of-range queries");
                paro_cost_t cost;
                bad += check(paro_cost(s, 7e9, 7e9, P, G, 8, 12, PARO_SCHED_DEFAULT, &cost) == PARO_OK, "paro_cost");
                paro_plan_destroy(pl);
            }
        }
    }
    // error paths of paro_plan itself
    paro_plan_t *pl = nullptr;
    int64_t one = 1, neg = -1, zero = 0;
    bad += check(paro_plan(0, 1, "GGG", &one, 1, nullptr, &pl) == PARO_EINVAL, "P = 0");
    bad += check(paro_plan(4, 3, "GGG", &one, 1, nullptr, &pl) == PARO_EINVAL, "G does not divide P");
    bad += check(paro_plan(4, 2, "GGG", &neg, 1, nullptr, &pl) == PARO_EINVAL, "negative size");
    bad += check(paro_plan(4, 2, "GGG", &zero, 1, nullptr, &pl) == PARO_EINVAL, "empty model");
    bad += check(paro_plan(4, 2, "GG", &one, 1, nullptr, &pl) != PARO_OK, "two letters");
    bad += check(paro_plan(4, 2, "GGGG", &one, 1, nullptr, &pl) != PARO_OK, "four letters");
    bad += check(paro_plan(4, 2, "GGG", nullptr, 1, nullptr, &pl) == PARO_EINVAL, "NULL sizes");
    bad += check(paro_plan(4, 2, nullptr, &one, 1, nullptr, &pl) != PARO_OK, "NULL strategy");
    bad += check(paro_plan(PARO_MAX_RANKS + 1, 1, "GGG", &one, 1, nullptr, &pl) == PARO_EINVAL, "too many ranks");
    paro_plan_opts_t o = {7, 0, nullptr, nullptr, PARO_BF16, 0};
    bad += check(paro_plan(4, 2, "GGG", &one, 1, &o, &pl) == PARO_EINVAL, "bad schedule kind");
    o = {PARO_SCHED_DEFAULT, 12, nullptr, nullptr, PARO_BF16, 0};
    bad += check(paro_plan(4, 2, "GGG", &one, 1, &o, &pl) == PARO_EINVAL, "alignment not a multiple of 8");
    bad += check(paro_two_step_saving(7e9, 64, 8, 8) == 7e9 * 7 * 7 / 64, "Eq. 1");
    std::printf("plans %ld, segments %ld, messages %ld, failures %d\n", plans, segs_total, msgs_total, bad);
    return bad ? 1 : 0;
}
