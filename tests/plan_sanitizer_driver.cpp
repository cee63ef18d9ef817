// Test driver: builds the host-side schedule builder with AddressSanitizer and
// UndefinedBehaviorSanitizer and pushes seeded random neighbourhoods through every
// algorithm.  Checks structural invariants only (results are checked elsewhere);
// the point is that the sanitizers see every code path.  Prints the number of plans.
#include <climits>
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
    // arguments that must be refused, never crash
    {
        iso::Comm c;
        int32_t one[1] = {4}, zero[1] = {0}, neg[2] = {3, -2}, big[3] = {2048, 2048, 1024}, off[1] = {1};
        int32_t many[ISO_MAX_DIMS + 1];
        for (auto &x : many) x = 1;
        REQUIRE(iso::build_comm(0, one, nullptr, 0, nullptr, c) == ISO_ERR_ARG);
        REQUIRE(iso::build_comm(ISO_MAX_DIMS + 1, many, nullptr, 0, nullptr, c) == ISO_ERR_ARG);
        REQUIRE(iso::build_comm(1, nullptr, nullptr, 0, nullptr, c) == ISO_ERR_ARG);
        REQUIRE(iso::build_comm(1, zero, nullptr, 0, nullptr, c) == ISO_ERR_ARG);
        REQUIRE(iso::build_comm(2, neg, nullptr, 0, nullptr, c) == ISO_ERR_ARG);
        REQUIRE(iso::build_comm(1, one, nullptr, -1, nullptr, c) == ISO_ERR_ARG);
        REQUIRE(iso::build_comm(1, one, nullptr, 1, nullptr, c) == ISO_ERR_ARG);
        REQUIRE(iso::build_comm(3, big, nullptr, 0, nullptr, c) == ISO_ERR_TOO_LARGE);      // 2^32 processes
        REQUIRE(iso::build_comm(ISO_MAX_DIMS, many, nullptr, 0, nullptr, c) == ISO_SUCCESS);
        REQUIRE(iso::build_comm(1, one, nullptr, 1, off, c) == ISO_SUCCESS);
        iso::Plan pl;
        REQUIRE(iso::build_plan(c, 2, ISO_ALG_COMBINED, pl) == ISO_ERR_ARG);
        REQUIRE(iso::build_plan(c, ISO_OP_ALLTOALL, 99, pl) == ISO_ERR_ARG);
        // extreme offsets: the reduction modulo the dimension size must not overflow
        int32_t dims2[2] = {7, 5}, ext[4] = {INT32_MAX, INT32_MIN, INT32_MIN, INT32_MAX};
        REQUIRE(iso::build_comm(2, dims2, nullptr, 2, ext, c) == ISO_SUCCESS);
        for (int i = 0; i < 2; ++i)
            for (int j = 0; j < 2; ++j) REQUIRE(c.c(i, j) >= 0 && c.c(i, j) < dims2[j]);
        for (int alg = 0; alg <= ISO_ALG_ONEHOP; ++alg)   // one hop per unit of coordinate would be 2^32 rounds
            for (int op = 0; op < 2; ++op)
                REQUIRE(iso::build_plan(c, op, alg, pl) == (alg == ISO_ALG_ONEHOP ? ISO_ERR_TOO_LARGE : ISO_SUCCESS));
    }
    std::printf("%ld\n", plans);
    return 0;
}
