// Test driver: the C ABI called from C++ with the HOST side of libiso (argument checks,
// schedule builder, binding, launch code) compiled under AddressSanitizer and
// UndefinedBehaviorSanitizer; the device code is the ordinary gfx950 build.  Seeded random
// tori, meshes, neighbourhoods and block sizes through every algorithm, regular and
// irregular, error paths included; every result is compared with the plain definition
// (recv[R][i] = send[R - C_i][i], Section 2) computed here on the host.
// Built by paper_1606_07676_amd.build.build_abi_sanitizer_driver(); run by tests/test_gpu_abi_sanitizer.py.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include <unistd.h>
#include "iso.h"
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1);} } while (0)
#define REQUIRE(c) do { if (!(c)) { fprintf(stderr, "FAILED line %d: %s\n", __LINE__, #c); exit(2); } } while (0)
static uint64_t state = 88172645463325252ull;
static uint32_t rnd(uint32_t n) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return (uint32_t)(state % n); }

static void ref(int d, const std::vector<int32_t> &dims, const std::vector<int32_t> &periodic, int s, const std::vector<int32_t> &rel,
                size_t m, bool allgather, const std::vector<uint8_t> &send, std::vector<uint8_t> &recv) {
    int64_t p = 1; for (int j = 0; j < d; ++j) p *= dims[j];
    std::vector<int64_t> co(d);
    for (int64_t R = 0; R < p; ++R) {
        int64_t rem = R; for (int j = d - 1; j >= 0; --j) { co[j] = rem % dims[j]; rem /= dims[j]; }
        for (int i = 0; i < s; ++i) {
            int64_t src = 0; bool ok = true;
            for (int j = 0; j < d; ++j) {
                int64_t t = co[j] - rel[(size_t)i * d + j];
                if (periodic[j]) { t %= dims[j]; if (t < 0) t += dims[j]; } else if (t < 0 || t >= dims[j]) ok = false;
                src = src * dims[j] + t;
            }
            if (!ok) continue;
            const uint8_t *sp = allgather ? &send[(size_t)src * m] : &send[((size_t)src * s + i) * m];
            memcpy(&recv[((size_t)R * s + i) * m], sp, m);
        }
    }
}

int main() {
    hipStream_t st; CK(hipStreamCreate(&st));
    long runs = 0;
    for (int iter = 0; iter < 60; ++iter) {
        const int d = 1 + (int)rnd(4);
        std::vector<int32_t> dims(d), periodic(d, 1);
        const bool mesh = iter % 3 == 2;
        for (int j = 0; j < d; ++j) { dims[j] = 1 + (int32_t)rnd(7); if (mesh) periodic[j] = (int32_t)rnd(2); }
        const int s = (int)rnd(iter % 10 == 0 ? 200 : 14);
        std::vector<int32_t> rel((size_t)s * d);
        for (auto &x : rel) x = (int32_t)rnd(9) - 4;
        const size_t ms[] = {0, 1, 16, 48, 100, 256};
        const size_t m = ms[rnd(6)];
        int64_t p = 1; for (int j = 0; j < d; ++j) p *= dims[j];
        iso_comm_t comm = nullptr;
        REQUIRE(iso_neighborhood_create_mesh(d, dims.data(), mesh ? periodic.data() : nullptr, s, rel.data(), &comm) == ISO_SUCCESS);
        iso_comm_info_t ci; REQUIRE(iso_neighborhood_info(comm, &ci) == ISO_SUCCESS && ci.p == p);
        for (int op = 0; op < 2; ++op) {
            const size_t send_bytes = (op == 0 ? (size_t)p * s : (size_t)p) * m, recv_bytes = (size_t)p * s * m;
            std::vector<uint8_t> send_h(send_bytes + 1), want(recv_bytes + 1, 0xEE), got(recv_bytes + 1);
            for (auto &b : send_h) b = (uint8_t)rnd(256);
            ref(d, dims, periodic, s, rel, m, op == 1, send_h, want);
            uint8_t *send_d, *recv_d; CK(hipMalloc(&send_d, send_bytes + 16)); CK(hipMalloc(&recv_d, recv_bytes + 16));
            CK(hipMemcpy(send_d, send_h.data(), send_bytes, hipMemcpyHostToDevice));
            for (int alg = 0; alg <= ISO_ALG_COMBINED_STAGED; ++alg) {
                size_t wsb = 0; int ws = iso_workspace_bytes(comm, op, alg, m, &wsb);
                if ((alg == ISO_ALG_ONEHOP || alg == ISO_ALG_COMBINED_STAGED) && mesh && ci.d > 0) {
                    bool any_np = false; for (int j = 0; j < d; ++j) any_np |= !periodic[j];
                    if (any_np) { REQUIRE(ws == ISO_ERR_ARG); continue; }
                }
                REQUIRE(ws == ISO_SUCCESS);
                uint8_t *work_d = nullptr; CK(hipMalloc(&work_d, wsb + 16));
                CK(hipMemset(recv_d, 0xEE, recv_bytes + 16));
                iso_request_t rq = nullptr;
                // error paths first
                if (wsb) { REQUIRE(iso_neighbor_alltoall_init(send_d, recv_d, m, work_d, wsb - 1, comm, alg, &rq) == ISO_ERR_WORKSPACE || op == 1); if (rq) iso_request_free(&rq); }
                if (recv_bytes && send_bytes) REQUIRE((op == 0 ? iso_neighbor_alltoall_init : iso_neighbor_allgather_init)(send_d, send_d, m, work_d, wsb, comm, alg, &rq) == ISO_ERR_OVERLAP);
                int ist = (op == 0 ? iso_neighbor_alltoall_init : iso_neighbor_allgather_init)(send_d, recv_d, m, work_d, wsb, comm, alg, &rq);
                REQUIRE(ist == ISO_SUCCESS);
                iso_request_info_t ri; REQUIRE(iso_request_info(rq, &ri) == ISO_SUCCESS);
                iso_plan_t pl; REQUIRE(iso_request_plan(rq, &pl) == ISO_SUCCESS);
                iso_plan_info_t pi; REQUIRE(iso_plan_info(pl, &pi) == ISO_SUCCESS);
                for (int r = 0; r < pi.launches; ++r) { iso_round_info_t rinfo; REQUIRE(iso_plan_round(pl, r, &rinfo) == ISO_SUCCESS); std::vector<iso_plan_entry_t> ent(rinfo.n_entries + 1); REQUIRE(iso_plan_entries(pl, r, ent.data(), rinfo.n_entries) == ISO_SUCCESS); }
                if (iter % 4 == 1) REQUIRE(iso_request_set_graph(rq, 1) == ISO_SUCCESS);
                REQUIRE(iso_start(rq, st) == ISO_SUCCESS);
                REQUIRE(iso_wait(rq) == ISO_SUCCESS);
                CK(hipMemcpy(got.data(), recv_d, recv_bytes, hipMemcpyDeviceToHost));
                REQUIRE(memcmp(got.data(), want.data(), recv_bytes) == 0);
                REQUIRE(iso_request_free(&rq) == ISO_SUCCESS && rq == nullptr);
                // the same collective on slot-major buffers: [s][p][m] instead of [p][s][m]
                if (recv_bytes) {
                    std::vector<uint8_t> send_sm(send_bytes + 1), want_sm(recv_bytes + 1), got_sm(recv_bytes + 1);
                    for (int64_t R = 0; R < p; ++R)
                        for (int i = 0; i < s; ++i) {
                            if (op == 0) memcpy(&send_sm[((size_t)i * p + R) * m], &send_h[((size_t)R * s + i) * m], m);
                            memcpy(&want_sm[((size_t)i * p + R) * m], &want[((size_t)R * s + i) * m], m);
                        }
                    if (op == 1) send_sm = send_h;
                    uint8_t *ssm_d, *rsm_d; CK(hipMalloc(&ssm_d, send_bytes + 16)); CK(hipMalloc(&rsm_d, recv_bytes + 16));
                    CK(hipMemcpy(ssm_d, send_sm.data(), send_bytes, hipMemcpyHostToDevice));
                    CK(hipMemset(rsm_d, 0xEE, recv_bytes + 16));
                    REQUIRE((op == 0 ? iso_neighbor_alltoall_init_layout : iso_neighbor_allgather_init_layout)(
                                ssm_d, rsm_d, m, ISO_LAYOUT_SLOT_MAJOR, work_d, wsb, comm, alg, &rq) == ISO_SUCCESS);
                    REQUIRE(iso_start(rq, st) == ISO_SUCCESS);
                    REQUIRE(iso_wait(rq) == ISO_SUCCESS);
                    CK(hipMemcpy(got_sm.data(), rsm_d, recv_bytes, hipMemcpyDeviceToHost));
                    REQUIRE(memcmp(got_sm.data(), want_sm.data(), recv_bytes) == 0);
                    REQUIRE(iso_request_free(&rq) == ISO_SUCCESS);
                    REQUIRE((op == 0 ? iso_neighbor_alltoall_init_layout : iso_neighbor_allgather_init_layout)(
                                ssm_d, rsm_d, m, 5, work_d, wsb, comm, alg, &rq) == ISO_ERR_ARG);
                    CK(hipFree(ssm_d)); CK(hipFree(rsm_d));
                    ++runs;
                }
                CK(hipFree(work_d));
                ++runs;
            }
            CK(hipFree(send_d)); CK(hipFree(recv_d));
        }
        // irregular: random sizes
        if (s > 0 && !mesh) {
            std::vector<size_t> sizes(s), sd(s), rd(s); size_t se = 0, re = 7;
            for (int i = 0; i < s; ++i) { sizes[i] = rnd(4) == 0 ? 0 : 1 + rnd(70); sd[i] = se; se += sizes[i] + rnd(3); }
            for (int i = s - 1; i >= 0; --i) { rd[i] = re; re += sizes[i] + rnd(5); }
            se += 1; re += 3;
            std::vector<uint8_t> send_h((size_t)p * se), want((size_t)p * re, 0xEE), got((size_t)p * re);
            for (auto &b : send_h) b = (uint8_t)rnd(256);
            std::vector<int64_t> co(d);
            for (int64_t R = 0; R < p; ++R) {
                int64_t rem = R; for (int j = d - 1; j >= 0; --j) { co[j] = rem % dims[j]; rem /= dims[j]; }
                for (int i = 0; i < s; ++i) { int64_t src = 0; for (int j = 0; j < d; ++j) { int64_t t = (co[j] - rel[(size_t)i * d + j]) % dims[j]; if (t < 0) t += dims[j]; src = src * dims[j] + t; }
                    memcpy(&want[(size_t)R * re + rd[i]], &send_h[(size_t)src * se + sd[i]], sizes[i]); }
            }
            uint8_t *send_d, *recv_d; CK(hipMalloc(&send_d, send_h.size() + 16)); CK(hipMalloc(&recv_d, want.size() + 16));
            CK(hipMemcpy(send_d, send_h.data(), send_h.size(), hipMemcpyHostToDevice));
            for (int alg = 0; alg <= ISO_ALG_COMBINED_STAGED; ++alg) {
                size_t wsb = 0; REQUIRE(iso_workspace_bytes_v(comm, 0, alg, sizes.data(), &wsb) == ISO_SUCCESS);
                uint8_t *work_d; CK(hipMalloc(&work_d, wsb + 16)); CK(hipMemset(recv_d, 0xEE, want.size()));
                iso_request_t rq = nullptr;
                REQUIRE(iso_neighbor_alltoallv_init(send_d, sizes.data(), sd.data(), se, recv_d, sizes.data(), rd.data(), re, work_d, wsb, comm, alg, &rq) == ISO_SUCCESS);
                REQUIRE(iso_start(rq, st) == ISO_SUCCESS); REQUIRE(iso_wait(rq) == ISO_SUCCESS);
                CK(hipMemcpy(got.data(), recv_d, want.size(), hipMemcpyDeviceToHost));
                REQUIRE(memcmp(got.data(), want.data(), want.size()) == 0);
                REQUIRE(iso_request_free(&rq) == ISO_SUCCESS); CK(hipFree(work_d)); ++runs;
            }
            CK(hipFree(send_d)); CK(hipFree(recv_d));
        }
        REQUIRE(iso_neighborhood_free(&comm) == ISO_SUCCESS && comm == nullptr);
        if (iter % 10 == 0) { printf("iter %d ok, %ld runs\n", iter, runs); fflush(stdout); }
    }
    // bad arguments
    iso_comm_t c = nullptr; int32_t dm[2] = {4, 0};
    REQUIRE(iso_neighborhood_create(2, dm, 0, nullptr, &c) == ISO_ERR_ARG && !c);
    REQUIRE(iso_neighborhood_create(0, dm, 0, nullptr, &c) == ISO_ERR_ARG);
    REQUIRE(iso_start(nullptr, nullptr) == ISO_ERR_ARG);
    printf("all ok: %ld collectives\n", runs);
    fflush(stdout);
    // Leave without running the HIP/HSA runtime's exit handlers: their teardown trips a check
    // inside the sanitizer's own device allocator that has nothing to do with the code under test.
    _exit(0);
}
