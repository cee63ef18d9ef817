// Test driver: builds the host-side schedule builder with AddressSanitizer and
// UndefinedBehaviorSanitizer and pushes seeded random neighbourhoods through every
// algorithm.  Checks structural invariants only (results are checked elsewhere);
// the point is that the sanitizers see every code path.  Prints the number of plans.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <set>
#include <utility>
#include <vector>

#include "iso_plan.hpp"

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(uint32_t n) {            // uniform in [0, n)
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)((state >> 33) % n);
}

#define REQUIRE(c) do { if (!(c)) { std::fprintf(stderr, "line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main() {
    long plans = 0;
    for (int iter = 0; iter < 600; ++iter) {
        const int d = 1 + (int)rnd(6);
        std::vector<int32_t> dims(d), periodic(d);
        const bool mesh = rnd(3) == 0;
        for (int j = 0; j < d; ++j) {
            dims[j] = 1 + (int32_t)rnd(iter % 7 == 0 ? 40 : 6);
            periodic[j] = mesh ? (int32_t)rnd(2) : 1;
        }
        const int s = (int)rnd(iter % 11 == 0 ? 300 : 30);
        const int span = 1 + (int)rnd(9);
        std::vector<int32_t> rel((size_t)s * d);
        for (auto &x : rel) x = (int32_t)rnd(2 * span + 1) - span;
        for (int i = 1; i < s; ++i)
            if (rnd(8) == 0)                   // repeat an earlier vector
                for (int j = 0; j < d; ++j) rel[(size_t)i * d + j] = rel[(size_t)rnd(i) * d + j];
        iso::Comm c;
        const int st = iso::build_comm(d, dims.data(), mesh ? periodic.data() : nullptr, s, rel.data(), c);
        if (st == ISO_ERR_TOO_LARGE) continue;
        REQUIRE(st == ISO_SUCCESS);
        (void)iso::allgather_dim_order(c, nullptr);
        for (int op = 0; op < 2; ++op)
            for (int alg = 0; alg <= ISO_ALG_ONEHOP; ++alg) {
                iso::Plan pl;
                const int ps = iso::build_plan(c, op, alg, pl);
                if (alg == ISO_ALG_ONEHOP && c.mesh) { REQUIRE(ps == ISO_ERR_ARG); continue; }
                REQUIRE(ps == ISO_SUCCESS);
                ++plans;
                std::set<std::pair<int, int>> final_writes;
                for (const iso::Round &r : pl.rounds) {
                    REQUIRE(!r.entries.empty());
                    std::set<std::pair<int, int>> w;
                    for (const iso_plan_entry_t &e : r.entries) {
                        REQUIRE(e.dst_buf == ISO_BUF_RECV || e.dst_buf == ISO_BUF_WORK);
                        REQUIRE(e.dst_buf != ISO_BUF_WORK || (e.dst_slot >= 0 && e.dst_slot < pl.work_slots));
                        REQUIRE(e.dst_buf != ISO_BUF_RECV || (e.dst_slot >= 0 && e.dst_slot < s));
                        REQUIRE(e.src_buf != ISO_BUF_WORK || (e.src_slot >= 0 && e.src_slot < pl.work_slots));
                        REQUIRE(e.ref >= 0 && e.ref < s);
                        REQUIRE(w.insert({e.dst_buf, e.dst_slot}).second);
                        if (e.dst_buf == ISO_BUF_RECV) final_writes.insert({e.dst_buf, e.dst_slot});
                    }
                }
                REQUIRE((int)final_writes.size() == s);
            }
    }
    std::printf("%ld\n", plans);
    return 0;
}
