// CPU-only test driver: the life cycle of communicators, plans and requests (every init call, both
// graph forms, starts, the allocation-free call, error paths that must release what they took)
// against the stand-in HIP runtime of hip_stub_runtime.cpp, under AddressSanitizer + LeakSanitizer.
// Ends with "lifecycle ok" only if the library left no device allocation and no graph object alive;
// host leaks are LeakSanitizer's to report at exit.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "iso.h"

extern "C" {
void *stub_device_alloc(size_t bytes);
void stub_device_free(void *q);
long stub_live_allocations(void);
long stub_live_graph_objects(void);
long stub_kernel_launches(void);
long stub_graph_launches(void);
long stub_graph_nodes(void);
}

#define REQUIRE(c) do { if (!(c)) { std::fprintf(stderr, "line %d: %s\n", __LINE__, #c); return 1; } } while (0)

static std::vector<int32_t> moore(int d, int r) {
    std::vector<int32_t> out, c((size_t)d, -r);
    for (;;) {
        bool zero = true;
        for (int x : c) zero = zero && x == 0;
        if (!zero) out.insert(out.end(), c.begin(), c.end());
        int j = d - 1;
        while (j >= 0 && c[(size_t)j] == r) c[(size_t)j--] = -r;
        if (j < 0) break;
        ++c[(size_t)j];
    }
    return out;
}

int main() {
    const int32_t dims[3] = {6, 5, 4}, mesh_flags[3] = {0, 1, 0};
    const std::vector<int32_t> offs = moore(3, 1);
    const int s = (int)offs.size() / 3;
    const size_t p = 120, m = 48;
    long requests = 0;
    for (int mesh = 0; mesh < 2; ++mesh) {
        iso_comm_t comm = nullptr;
        REQUIRE(iso_neighborhood_create_mesh(3, dims, mesh ? mesh_flags : nullptr, s, offs.data(), &comm) == ISO_SUCCESS);
        iso_comm_info_t ci;
        REQUIRE(iso_neighborhood_info(comm, &ci) == ISO_SUCCESS && ci.s == s);
        for (int op = 0; op < 2; ++op)
            for (int alg = 0; alg <= ISO_ALG_ONEHOP; ++alg) {
                if (mesh && alg == ISO_ALG_ONEHOP) continue;
                iso_plan_t plan = nullptr;
                REQUIRE(iso_plan_create(comm, op, alg, &plan) == ISO_SUCCESS);
                iso_plan_info_t pi;
                REQUIRE(iso_plan_info(plan, &pi) == ISO_SUCCESS);
                REQUIRE(iso_plan_free(&plan) == ISO_SUCCESS && plan == nullptr);
                size_t wsb = 0;
                REQUIRE(iso_workspace_bytes(comm, op, alg, m, &wsb) == ISO_SUCCESS);
                void *send = stub_device_alloc(p * (size_t)s * m), *recv = stub_device_alloc(p * (size_t)s * m);
                void *work = stub_device_alloc(wsb + 16);
                REQUIRE(send && recv && work);
                // regular, both layouts
                for (int layout = 0; layout < 2; ++layout) {
                    iso_request_t req = nullptr;
                    int st = op == ISO_OP_ALLTOALL
                                 ? iso_neighbor_alltoall_init_layout(send, recv, m, layout, work, wsb, comm, alg, &req)
                                 : iso_neighbor_allgather_init_layout(send, recv, m, layout, work, wsb, comm, alg, &req);
                    REQUIRE(st == ISO_SUCCESS && req);
                    ++requests;
                    REQUIRE(iso_start(req, nullptr) == ISO_SUCCESS);
                    for (int form = ISO_GRAPH_CHAIN; form <= ISO_GRAPH_BRANCHES; ++form) {
                        REQUIRE(iso_request_set_graph(req, form) == ISO_SUCCESS);
                        REQUIRE(iso_start(req, nullptr) == ISO_SUCCESS);
                    }
                    if (layout) REQUIRE(iso_request_set_graph(req, ISO_GRAPH_OFF) == ISO_SUCCESS);
                    iso_request_info_t ri;
                    REQUIRE(iso_request_info(req, &ri) == ISO_SUCCESS);
                    REQUIRE(iso_start_range(req, 0, ri.launches, nullptr) == ISO_SUCCESS);
                    iso_plan_t view = nullptr;
                    REQUIRE(iso_request_plan(req, &view) == ISO_SUCCESS && view);
                    REQUIRE(iso_wait(req) == ISO_SUCCESS);
                    REQUIRE(iso_request_free(&req) == ISO_SUCCESS && req == nullptr);
                }
                // irregular: per-neighbour sizes, rows with a gap
                if (op == ISO_OP_ALLTOALL) {
                    std::vector<size_t> sizes((size_t)s), displs((size_t)s);
                    size_t at = 0;
                    for (int i = 0; i < s; ++i) {
                        sizes[(size_t)i] = (size_t)(i % 5 == 0 ? 0 : 1 + (i * 7) % 40);
                        displs[(size_t)i] = at;
                        at += sizes[(size_t)i] + 3;
                    }
                    REQUIRE(at <= (size_t)s * m);
                    size_t wv = 0;
                    REQUIRE(iso_workspace_bytes_v(comm, op, alg, sizes.data(), &wv) == ISO_SUCCESS);
                    void *workv = stub_device_alloc(wv + 16);
                    iso_request_t req = nullptr;
                    REQUIRE(iso_neighbor_alltoallw_init(send, sizes.data(), displs.data(), at, recv, sizes.data(),
                                                        displs.data(), at, workv, wv, comm, alg, &req) == ISO_SUCCESS);
                    ++requests;
                    REQUIRE(iso_request_set_graph(req, ISO_GRAPH_BRANCHES) == ISO_SUCCESS);
                    REQUIRE(iso_start(req, nullptr) == ISO_SUCCESS);
                    REQUIRE(iso_request_free(&req) == ISO_SUCCESS);
                    // an error after the plan was built: a workspace that is too small releases everything
                    if (wv) {
                        REQUIRE(iso_neighbor_alltoallv_init(send, sizes.data(), displs.data(), at, recv, sizes.data(),
                                                            displs.data(), at, workv, wv - 1, comm, alg, &req) ==
                                ISO_ERR_WORKSPACE);
                        REQUIRE(req == nullptr);
                    }
                    stub_device_free(workv);
                }
                // overlap and bad pointers are refused without leaving anything behind
                if (op == ISO_OP_ALLTOALL) {
                    iso_request_t bad = nullptr;
                    REQUIRE(iso_neighbor_alltoall_init(send, send, m, work, wsb, comm, alg, &bad) == ISO_ERR_OVERLAP);
                    int dummy[4];
                    REQUIRE(iso_neighbor_alltoall_init(dummy, recv, m, work, wsb, comm, alg, &bad) == ISO_ERR_POINTER);
                    REQUIRE(bad == nullptr);
                }
                stub_device_free(send);
                stub_device_free(recv);
                stub_device_free(work);
            }
        // the straightforward algorithm under its own names, and the allocation-free call
        void *send = stub_device_alloc(p * (size_t)s * m), *recv = stub_device_alloc(p * (size_t)s * m);
        iso_request_t req = nullptr;
        REQUIRE(iso_neighbor_alltoall_sx_init(send, recv, m, ISO_SX_FUSED, comm, &req) == ISO_SUCCESS);
        REQUIRE(iso_start(req, nullptr) == ISO_SUCCESS && iso_request_free(&req) == ISO_SUCCESS);
        REQUIRE(iso_neighbor_allgather_sx_init(send, recv, m, ISO_SX_LAUNCHES, comm, &req) == ISO_SUCCESS);
        REQUIRE(iso_request_free(&req) == ISO_SUCCESS);
        requests += 2;
        const long live_before = stub_live_allocations();
        REQUIRE(iso_neighbor_alltoall_noalloc(send, recv, m, comm, ISO_ALG_COMBINED, nullptr) == ISO_SUCCESS);
        REQUIRE(iso_neighbor_alltoall_noalloc(send, recv, (size_t)1 << 20, comm, ISO_ALG_COMBINED, nullptr) != ISO_SUCCESS);
        REQUIRE(stub_live_allocations() == live_before);       // it allocates nothing
        stub_device_free(send);
        stub_device_free(recv);
        REQUIRE(iso_neighborhood_free(&comm) == ISO_SUCCESS && comm == nullptr);
    }
    REQUIRE(stub_kernel_launches() > 0 && stub_graph_launches() > 0 && stub_graph_nodes() > 0);
    if (stub_live_allocations() != 0 || stub_live_graph_objects() != 0) {
        std::fprintf(stderr, "left behind: %ld device allocations, %ld graph objects\n", stub_live_allocations(),
                     stub_live_graph_objects());
        return 2;
    }
    std::printf("lifecycle ok: %ld requests, %ld kernel launches, %ld graph launches\n", requests,
                stub_kernel_launches(), stub_graph_launches());
    return 0;
}
