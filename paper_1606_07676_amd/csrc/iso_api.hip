// C ABI of libiso (see include/iso.h): handles, argument checks and the launch
// of a bound request's rounds.  The binding of a schedule to buffers lives in
// iso_bind.hpp, the schedules in iso_plan.cpp, the kernels in iso_kernels.hpp.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "iso.h"
#include "iso_bind.hpp"
#include "iso_kernels.hpp"
#include "iso_plan.hpp"

namespace iso {
thread_local int g_last_hip_error = 0;
}

// Device memory for iso_neighbor_alltoall_noalloc: the table of block index maps in the first
// ISO_NOALLOC_TABLE_BYTES, the intermediate buffer of Algorithm 1 in the rest.  Every device the
// library's code is loaded on holds its own copy until the process ends.  In host code the name
// only stands for the symbol: the address on the current device comes from hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[ISO_NOALLOC_SCRATCH_BYTES];

struct iso_comm_s {
    iso::Comm c;
    int64_t allgather_moves = -1;        // computed by the first iso_neighborhood_info
};

struct iso_plan_s {
    iso::Plan p;
};

struct iso_request_s {
    iso::BoundRequest b;
    iso_plan_s plan_view;                // what iso_request_plan hands out
    hipStream_t last_stream = nullptr;
    bool started = false;
    hipGraph_t graph = nullptr;          // the launches of one collective as a HIP graph
    hipGraphExec_t graph_exec = nullptr;
    int graph_form = 0;                  // ISO_GRAPH_CHAIN or ISO_GRAPH_BRANCHES: what `graph` was built as
    bool use_graph = false;
};

namespace {

using iso::g_last_hip_error;

template <typename F>
int guarded(F &&f) {
    try {
        return f();
    } catch (const std::bad_alloc &) {
        return ISO_ERR_NOMEM;
    } catch (...) {
        return ISO_ERR_ARG;
    }
}

// p times the sum of the block sizes must stay far inside 64 bits (all later address and
// workspace arithmetic relies on it).
bool sizes_too_large(const iso::Comm &c, const std::vector<uint64_t> &sizes) {
    const uint64_t limit = (~uint64_t(0) >> 2) / (uint64_t)std::max<int64_t>(1, c.p);
    uint64_t sum = 0;
    for (uint64_t sz : sizes) {
        if (sz > limit || sum > limit - sz) return true;
        sum += sz;
    }
    return false;
}

// Regular blocks of m bytes.  Rank-major: a process's s blocks back to back in neighbour
// order, [p][s][m].  Slot-major: one plane of p blocks per neighbour, [s][p][m]; the
// distance between consecutive ranks is then m and block i starts i*p*m into the buffer.
iso::Layout regular_layout(const iso::Comm &c, int op, size_t m, int layout = ISO_LAYOUT_RANK_MAJOR) {
    iso::Layout lay;
    const size_t s = (size_t)c.s;
    const uint64_t slot = layout == ISO_LAYOUT_SLOT_MAJOR ? (uint64_t)c.p * m : m;
    lay.slot_major = layout == ISO_LAYOUT_SLOT_MAJOR;
    lay.size.assign(s, m);
    lay.send_displ.resize(s);
    lay.recv_displ.resize(s);
    for (size_t i = 0; i < s; ++i) {
        lay.send_displ[i] = op == ISO_OP_ALLTOALL ? i * slot : 0;
        lay.recv_displ[i] = i * slot;
    }
    const uint64_t row = lay.slot_major ? m : s * m;           // bytes between consecutive ranks
    const uint64_t span = s ? (s - 1) * slot + m : 0;           // first to last byte of one rank's blocks
    lay.send_extent = op == ISO_OP_ALLTOALL ? row : (s ? m : 0);
    lay.send_span = op == ISO_OP_ALLTOALL ? span : (s ? m : 0);
    lay.recv_extent = row;
    lay.recv_span = span;
    return lay;
}

// Blocks of a row must lie inside the row's extent; receive blocks must not overlap.
int check_rows(const std::vector<uint64_t> &size, const std::vector<uint64_t> &displ, uint64_t extent,
               bool disjoint, uint64_t &span) {
    span = 0;
    std::vector<std::pair<uint64_t, uint64_t>> iv;
    for (size_t i = 0; i < size.size(); ++i) {
        if (!size[i]) continue;
        if (displ[i] > extent || size[i] > extent - displ[i]) return ISO_ERR_ARG;
        span = std::max(span, displ[i] + size[i]);
        iv.emplace_back(displ[i], displ[i] + size[i]);
    }
    if (disjoint) {
        std::sort(iv.begin(), iv.end());
        for (size_t q = 1; q < iv.size(); ++q)
            if (iv[q].first < iv[q - 1].second) return ISO_ERR_OVERLAP;
    }
    return ISO_SUCCESS;
}

int make_request(int op, const iso::Layout &lay, const void *sendbuf, void *recvbuf, void *workspace,
                 size_t workspace_bytes, iso_comm_t comm, int algorithm, iso_request_t *out) {
    iso_request_s *rq = new iso_request_s();
    struct Guard {
        iso_request_s *r;
        ~Guard() {
            if (r) {
                if (r->b.dev_table) (void)hipFree(r->b.dev_table);
                delete r;
            }
        }
    } guard{rq};
    int st = iso::build_plan(comm->c, op, algorithm, rq->b.plan);
    if (st != ISO_SUCCESS) return st;
    st = iso::bind_request(rq->b, comm->c, lay, sendbuf, recvbuf, workspace, workspace_bytes);
    if (st != ISO_SUCCESS) return st;
    guard.r = nullptr;
    *out = rq;
    return ISO_SUCCESS;
}

int init_regular(int op, const void *sendbuf, void *recvbuf, size_t m, int layout, void *workspace,
                 size_t workspace_bytes, iso_comm_t comm, int algorithm, iso_request_t *out) {
    if (!out) return ISO_ERR_ARG;
    *out = nullptr;
    if (!comm || (layout != ISO_LAYOUT_RANK_MAJOR && layout != ISO_LAYOUT_SLOT_MAJOR)) return ISO_ERR_ARG;
    const uint64_t p = (uint64_t)comm->c.p, s = (uint64_t)comm->c.s;
    if (m && p > (~(uint64_t)0 >> 2) / std::max<uint64_t>(1, s) / m) return ISO_ERR_TOO_LARGE;
    return make_request(op, regular_layout(comm->c, op, m, layout), sendbuf, recvbuf, workspace,
                        workspace_bytes, comm, algorithm, out);
}

// Planes of a slot-major irregular buffer: plane i holds block i of all p ranks back to back,
// [displ_i, displ_i + p * size_i).  Receive planes must not overlap.
int check_planes(const std::vector<uint64_t> &size, const std::vector<uint64_t> &displ, uint64_t p, bool disjoint) {
    const uint64_t limit = ~uint64_t(0) >> 2;
    std::vector<std::pair<uint64_t, uint64_t>> iv;
    for (size_t i = 0; i < size.size(); ++i) {
        if (!size[i]) continue;
        if (size[i] > limit / std::max<uint64_t>(1, p) || displ[i] > limit) return ISO_ERR_TOO_LARGE;
        iv.emplace_back(displ[i], displ[i] + p * size[i]);
    }
    if (disjoint) {
        std::sort(iv.begin(), iv.end());
        for (size_t q = 1; q < iv.size(); ++q)
            if (iv[q].first < iv[q - 1].second) return ISO_ERR_OVERLAP;
    }
    return ISO_SUCCESS;
}

int init_alltoallv(const void *sendbuf, const size_t *send_sizes, const size_t *send_displs, size_t send_extent,
                   void *recvbuf, const size_t *recv_sizes, const size_t *recv_displs, size_t recv_extent,
                   int layout, void *workspace, size_t workspace_bytes, iso_comm_t comm, int algorithm,
                   iso_request_t *req) {
    if (!req) return ISO_ERR_ARG;
    *req = nullptr;
    if (!comm || (layout != ISO_LAYOUT_RANK_MAJOR && layout != ISO_LAYOUT_SLOT_MAJOR)) return ISO_ERR_ARG;
    const size_t s = (size_t)comm->c.s;
    if (s && (!send_sizes || !send_displs || !recv_sizes || !recv_displs)) return ISO_ERR_ARG;
    iso::Layout lay;
    lay.size.assign(send_sizes, send_sizes + s);
    lay.send_displ.assign(send_displs, send_displs + s);
    lay.recv_displ.assign(recv_displs, recv_displs + s);
    for (size_t i = 0; i < s; ++i)
        if (send_sizes[i] != recv_sizes[i]) return ISO_ERR_ARG;      // sizes must match pairwise
    lay.send_extent = send_extent;
    lay.recv_extent = recv_extent;
    lay.slot_major = layout == ISO_LAYOUT_SLOT_MAJOR;
    int st;
    if (lay.slot_major) {
        if ((st = check_planes(lay.size, lay.send_displ, (uint64_t)comm->c.p, false)) != ISO_SUCCESS) return st;
        if ((st = check_planes(lay.size, lay.recv_displ, (uint64_t)comm->c.p, true)) != ISO_SUCCESS) return st;
    } else {
        if ((st = check_rows(lay.size, lay.send_displ, send_extent, false, lay.send_span)) != ISO_SUCCESS) return st;
        if ((st = check_rows(lay.size, lay.recv_displ, recv_extent, true, lay.recv_span)) != ISO_SUCCESS) return st;
    }
    return make_request(ISO_OP_ALLTOALL, lay, sendbuf, recvbuf, workspace, workspace_bytes, comm, algorithm, req);
}

int init_allgatherv(const void *sendbuf, size_t send_size, size_t send_extent, void *recvbuf,
                    const size_t *recv_sizes, const size_t *recv_displs, size_t recv_extent, int layout,
                    void *workspace, size_t workspace_bytes, iso_comm_t comm, int algorithm, iso_request_t *req) {
    if (!req) return ISO_ERR_ARG;
    *req = nullptr;
    if (!comm || (layout != ISO_LAYOUT_RANK_MAJOR && layout != ISO_LAYOUT_SLOT_MAJOR)) return ISO_ERR_ARG;
    const size_t s = (size_t)comm->c.s;
    if (s && (!recv_sizes || !recv_displs)) return ISO_ERR_ARG;
    iso::Layout lay;
    lay.size.assign(s, send_size);
    lay.send_displ.assign(s, 0);
    lay.recv_displ.assign(recv_displs, recv_displs + s);
    for (size_t i = 0; i < s; ++i)
        if (recv_sizes[i] != send_size) return ISO_ERR_ARG;         // every process sends one size
    lay.send_extent = send_extent;
    lay.recv_extent = recv_extent;
    lay.slot_major = layout == ISO_LAYOUT_SLOT_MAJOR;
    if (s && send_size > send_extent) return ISO_ERR_ARG;
    lay.send_span = s ? send_size : 0;
    int st;
    if (lay.slot_major) {
        if ((st = check_planes(lay.size, lay.recv_displ, (uint64_t)comm->c.p, true)) != ISO_SUCCESS) return st;
    } else {
        if ((st = check_rows(lay.size, lay.recv_displ, recv_extent, true, lay.recv_span)) != ISO_SUCCESS) return st;
    }
    return make_request(ISO_OP_ALLGATHER, lay, sendbuf, recvbuf, workspace, workspace_bytes, comm, algorithm, req);
}

// Address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char *g_scratch_ptr[kMaxDevices] = {};

int scratch_of_current_device(unsigned char **out) {
    int dev = -1;
    ISO_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ISO_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        ISO_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return ISO_ERR_HIP;
        g_scratch_ptr[dev] = (unsigned char *)ptr;
    }
    *out = g_scratch_ptr[dev];
    return ISO_SUCCESS;
}

}  // namespace

extern "C" {

int iso_neighborhood_create(int d, const int32_t *dims, int s, const int32_t *rel_coords,
                            iso_comm_t *comm) {
    return iso_neighborhood_create_mesh(d, dims, nullptr, s, rel_coords, comm);
}

int iso_neighborhood_create_mesh(int d, const int32_t *dims, const int32_t *periodic, int s,
                                 const int32_t *rel_coords, iso_comm_t *comm) {
    return guarded([&]() -> int {
        if (!comm) return ISO_ERR_ARG;
        *comm = nullptr;
        iso_comm_s *h = new iso_comm_s();
        int st = iso::build_comm(d, dims, periodic, s, rel_coords, h->c);
        if (st != ISO_SUCCESS) {
            delete h;
            return st;
        }
        *comm = h;
        return ISO_SUCCESS;
    });
}

int iso_neighborhood_info(iso_comm_t comm, iso_comm_info_t *info) {
    return guarded([&]() -> int {
        if (!comm || !info) return ISO_ERR_ARG;
        const iso::Comm &c = comm->c;
        if (comm->allgather_moves < 0) (void)iso::allgather_dim_order(c, &comm->allgather_moves);
        info->d = c.d;
        info->s = c.s;
        info->p = c.p;
        info->rounds = c.rounds();
        info->self_slots = 0;
        info->alltoall_moves = 0;
        for (int i = 0; i < c.s; ++i) {
            const int n = c.nnz(i);
            info->alltoall_moves += n;
            info->self_slots += n == 0;
        }
        info->allgather_moves = comm->allgather_moves;
        return ISO_SUCCESS;
    });
}

int iso_neighborhood_free(iso_comm_t *comm) {
    if (!comm) return ISO_ERR_ARG;
    delete *comm;
    *comm = nullptr;
    return ISO_SUCCESS;
}

int iso_plan_create(iso_comm_t comm, int op, int algorithm, iso_plan_t *plan) {
    return guarded([&]() -> int {
        if (!plan) return ISO_ERR_ARG;
        *plan = nullptr;
        if (!comm) return ISO_ERR_ARG;
        iso_plan_s *h = new iso_plan_s();
        int st = iso::build_plan(comm->c, op, algorithm, h->p);
        if (st != ISO_SUCCESS) {
            delete h;
            return st;
        }
        *plan = h;
        return ISO_SUCCESS;
    });
}

int iso_plan_info(iso_plan_t plan, iso_plan_info_t *info) {
    if (!plan || !info) return ISO_ERR_ARG;
    const iso::Plan &p = plan->p;
    std::memset(info, 0, sizeof(*info));
    info->op = p.op;
    info->algorithm = p.algorithm;
    info->launches = (int32_t)p.rounds.size();
    info->work_slots = p.work_slots;
    info->entries = p.entries();
    for (size_t j = 0; j < p.dim_order.size() && j < ISO_MAX_DIMS; ++j) info->dim_order[j] = p.dim_order[j];
    return ISO_SUCCESS;
}

int iso_plan_round(iso_plan_t plan, int round, iso_round_info_t *info) {
    if (!plan || !info || round < 0 || (size_t)round >= plan->p.rounds.size()) return ISO_ERR_ARG;
    const iso::Round &r = plan->p.rounds[(size_t)round];
    info->kind = r.kind;
    info->dim = r.kind == ISO_ROUND_SHIFT ? r.dim : -1;
    info->n_entries = (int32_t)r.entries.size();
    info->reserved = 0;
    return ISO_SUCCESS;
}

int iso_plan_entries(iso_plan_t plan, int round, iso_plan_entry_t *out, int capacity) {
    if (!plan || round < 0 || (size_t)round >= plan->p.rounds.size() || capacity < 0 ||
        (capacity > 0 && !out))
        return ISO_ERR_ARG;
    const iso::Round &r = plan->p.rounds[(size_t)round];
    const size_t n = std::min<size_t>((size_t)capacity, r.entries.size());
    if (n) std::memcpy(out, r.entries.data(), n * sizeof(iso_plan_entry_t));
    return ISO_SUCCESS;
}

int iso_plan_free(iso_plan_t *plan) {
    if (!plan) return ISO_ERR_ARG;
    delete *plan;
    *plan = nullptr;
    return ISO_SUCCESS;
}

int iso_workspace_bytes(iso_comm_t comm, int op, int algorithm, size_t m, size_t *bytes) {
    return guarded([&]() -> int {
        if (!comm || !bytes) return ISO_ERR_ARG;
        iso::Plan pl;
        int st = iso::build_plan(comm->c, op, algorithm, pl);
        if (st != ISO_SUCCESS) return st;
        if (sizes_too_large(comm->c, std::vector<uint64_t>((size_t)comm->c.s, m))) return ISO_ERR_TOO_LARGE;
        *bytes = (size_t)iso::work_layout(pl, regular_layout(comm->c, op, m)).bytes;
        return ISO_SUCCESS;
    });
}

int iso_alltoall_workspace_bytes(iso_comm_t comm, size_t m, size_t *bytes) {
    return iso_workspace_bytes(comm, ISO_OP_ALLTOALL, ISO_ALG_COMBINED, m, bytes);
}

int iso_allgather_workspace_bytes(iso_comm_t comm, size_t m, size_t *bytes) {
    return iso_workspace_bytes(comm, ISO_OP_ALLGATHER, ISO_ALG_COMBINED, m, bytes);
}

int iso_workspace_bytes_v(iso_comm_t comm, int op, int algorithm, const size_t *sizes, size_t *bytes) {
    return guarded([&]() -> int {
        if (!comm || !bytes || (comm->c.s > 0 && !sizes)) return ISO_ERR_ARG;
        iso::Plan pl;
        int st = iso::build_plan(comm->c, op, algorithm, pl);
        if (st != ISO_SUCCESS) return st;
        iso::Layout lay;
        lay.size.assign(sizes, sizes + comm->c.s);
        if (op == ISO_OP_ALLGATHER)                       // every process sends one size
            for (int i = 1; i < comm->c.s; ++i)
                if (sizes[i] != sizes[0]) return ISO_ERR_ARG;
        if (sizes_too_large(comm->c, lay.size)) return ISO_ERR_TOO_LARGE;
        *bytes = (size_t)iso::work_layout(pl, lay).bytes;
        return ISO_SUCCESS;
    });
}

int iso_neighbor_alltoall_init(const void *sendbuf, void *recvbuf, size_t m, void *workspace,
                               size_t workspace_bytes, iso_comm_t comm, int algorithm,
                               iso_request_t *req) {
    return guarded([&]() -> int {
        return init_regular(ISO_OP_ALLTOALL, sendbuf, recvbuf, m, ISO_LAYOUT_RANK_MAJOR, workspace,
                            workspace_bytes, comm, algorithm, req);
    });
}

int iso_neighbor_allgather_init(const void *sendbuf, void *recvbuf, size_t m, void *workspace,
                                size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                iso_request_t *req) {
    return guarded([&]() -> int {
        return init_regular(ISO_OP_ALLGATHER, sendbuf, recvbuf, m, ISO_LAYOUT_RANK_MAJOR, workspace,
                            workspace_bytes, comm, algorithm, req);
    });
}

int iso_neighbor_alltoall_sx_init(const void *sendbuf, void *recvbuf, size_t m, int mode, iso_comm_t comm,
                                  iso_request_t *req) {
    return guarded([&]() -> int {
        if (req) *req = nullptr;
        if (mode != ISO_SX_LAUNCHES && mode != ISO_SX_FUSED) return ISO_ERR_ARG;
        return init_regular(ISO_OP_ALLTOALL, sendbuf, recvbuf, m, ISO_LAYOUT_RANK_MAJOR, nullptr, 0, comm,
                            mode == ISO_SX_FUSED ? ISO_ALG_SX_FUSED : ISO_ALG_SX_ROUNDS, req);
    });
}

int iso_neighbor_allgather_sx_init(const void *sendbuf, void *recvbuf, size_t m, int mode, iso_comm_t comm,
                                   iso_request_t *req) {
    return guarded([&]() -> int {
        if (req) *req = nullptr;
        if (mode != ISO_SX_LAUNCHES && mode != ISO_SX_FUSED) return ISO_ERR_ARG;
        return init_regular(ISO_OP_ALLGATHER, sendbuf, recvbuf, m, ISO_LAYOUT_RANK_MAJOR, nullptr, 0, comm,
                            mode == ISO_SX_FUSED ? ISO_ALG_SX_FUSED : ISO_ALG_SX_ROUNDS, req);
    });
}

int iso_neighbor_alltoall_init_layout(const void *sendbuf, void *recvbuf, size_t m, int layout,
                                      void *workspace, size_t workspace_bytes, iso_comm_t comm,
                                      int algorithm, iso_request_t *req) {
    return guarded([&]() -> int {
        return init_regular(ISO_OP_ALLTOALL, sendbuf, recvbuf, m, layout, workspace, workspace_bytes, comm,
                            algorithm, req);
    });
}

int iso_neighbor_allgather_init_layout(const void *sendbuf, void *recvbuf, size_t m, int layout,
                                       void *workspace, size_t workspace_bytes, iso_comm_t comm,
                                       int algorithm, iso_request_t *req) {
    return guarded([&]() -> int {
        return init_regular(ISO_OP_ALLGATHER, sendbuf, recvbuf, m, layout, workspace, workspace_bytes, comm,
                            algorithm, req);
    });
}

int iso_neighbor_alltoallv_init(const void *sendbuf, const size_t *send_sizes, const size_t *send_displs,
                                size_t send_extent, void *recvbuf, const size_t *recv_sizes,
                                const size_t *recv_displs, size_t recv_extent, void *workspace,
                                size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                iso_request_t *req) {
    return guarded([&]() -> int {
        return init_alltoallv(sendbuf, send_sizes, send_displs, send_extent, recvbuf, recv_sizes, recv_displs,
                              recv_extent, ISO_LAYOUT_RANK_MAJOR, workspace, workspace_bytes, comm, algorithm, req);
    });
}

int iso_neighbor_allgatherv_init(const void *sendbuf, size_t send_size, size_t send_extent, void *recvbuf,
                                 const size_t *recv_sizes, const size_t *recv_displs, size_t recv_extent,
                                 void *workspace, size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                 iso_request_t *req) {
    return guarded([&]() -> int {
        return init_allgatherv(sendbuf, send_size, send_extent, recvbuf, recv_sizes, recv_displs, recv_extent,
                               ISO_LAYOUT_RANK_MAJOR, workspace, workspace_bytes, comm, algorithm, req);
    });
}

int iso_neighbor_alltoallv_init_layout(const void *sendbuf, const size_t *send_sizes, const size_t *send_displs,
                                       size_t send_extent, void *recvbuf, const size_t *recv_sizes,
                                       const size_t *recv_displs, size_t recv_extent, int layout,
                                       void *workspace, size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                       iso_request_t *req) {
    return guarded([&]() -> int {
        return init_alltoallv(sendbuf, send_sizes, send_displs, send_extent, recvbuf, recv_sizes, recv_displs,
                              recv_extent, layout, workspace, workspace_bytes, comm, algorithm, req);
    });
}

int iso_neighbor_allgatherv_init_layout(const void *sendbuf, size_t send_size, size_t send_extent, void *recvbuf,
                                        const size_t *recv_sizes, const size_t *recv_displs, size_t recv_extent,
                                        int layout, void *workspace, size_t workspace_bytes, iso_comm_t comm,
                                        int algorithm, iso_request_t *req) {
    return guarded([&]() -> int {
        return init_allgatherv(sendbuf, send_size, send_extent, recvbuf, recv_sizes, recv_displs, recv_extent,
                               layout, workspace, workspace_bytes, comm, algorithm, req);
    });
}

int iso_neighbor_alltoallw_init(const void *sendbuf, const size_t *send_sizes, const size_t *send_displs,
                                size_t send_extent, void *recvbuf, const size_t *recv_sizes,
                                const size_t *recv_displs, size_t recv_extent, void *workspace,
                                size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                iso_request_t *req) {
    return iso_neighbor_alltoallv_init(sendbuf, send_sizes, send_displs, send_extent, recvbuf, recv_sizes,
                                       recv_displs, recv_extent, workspace, workspace_bytes, comm, algorithm,
                                       req);
}

int iso_neighbor_allgatherw_init(const void *sendbuf, size_t send_size, size_t send_extent, void *recvbuf,
                                 const size_t *recv_sizes, const size_t *recv_displs, size_t recv_extent,
                                 void *workspace, size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                 iso_request_t *req) {
    return iso_neighbor_allgatherv_init(sendbuf, send_size, send_extent, recvbuf, recv_sizes, recv_displs,
                                        recv_extent, workspace, workspace_bytes, comm, algorithm, req);
}

int iso_neighbor_alltoall_noalloc(const void *sendbuf, void *recvbuf, size_t m, iso_comm_t comm,
                                  int algorithm, void *hip_stream) {
    return guarded([&]() -> int {
        if (!comm) return ISO_ERR_ARG;
        const uint64_t p = (uint64_t)comm->c.p, s = (uint64_t)comm->c.s;
        if (m && p > (~(uint64_t)0 >> 2) / std::max<uint64_t>(1, s) / m) return ISO_ERR_TOO_LARGE;
        unsigned char *ptr = nullptr;
        int st = scratch_of_current_device(&ptr);
        if (st != ISO_SUCCESS) return st;
        hipStream_t stream = (hipStream_t)hip_stream;
        iso::BoundRequest b;
        if ((st = iso::build_plan(comm->c, ISO_OP_ALLTOALL, algorithm, b.plan)) != ISO_SUCCESS) return st;
        const iso::StaticArena arena{ptr, ISO_NOALLOC_TABLE_BYTES, stream};
        st = iso::bind_request(b, comm->c, regular_layout(comm->c, ISO_OP_ALLTOALL, m), sendbuf, recvbuf,
                               ptr + ISO_NOALLOC_TABLE_BYTES, ISO_NOALLOC_SCRATCH_BYTES - ISO_NOALLOC_TABLE_BYTES,
                               &arena);
        if (st != ISO_SUCCESS) return st;
        for (const iso::Launch &l : b.launches)
            if ((st = iso::enqueue(b.info.vector_bytes, l, stream)) != ISO_SUCCESS) return st;
        return ISO_SUCCESS;
    });
}

int iso_request_set_graph(iso_request_t req, int enable) {
    if (!req || enable < 0 || enable > ISO_GRAPH_BRANCHES) return ISO_ERR_ARG;
    if (!enable || req->b.launches.empty()) {
        req->use_graph = false;
        return ISO_SUCCESS;
    }
    if (req->graph_exec && req->graph_form != enable) {       // the other form was built before: replace it
        ISO_HIP_TRY(hipStreamSynchronize(req->last_stream));
        (void)hipGraphExecDestroy(req->graph_exec);
        (void)hipGraphDestroy(req->graph);
        req->graph_exec = nullptr;
        req->graph = nullptr;
    }
    if (!req->graph_exec) {
        // One kernel node per launch.  ISO_GRAPH_CHAIN: every node after the one before it.
        // ISO_GRAPH_BRANCHES: an edge from an earlier launch only where the two touch a common block and
        // one of them writes it (the send buffer is never written): the rounds of one dimension move
        // disjoint blocks and become parallel branches, a round of the next dimension waits only for the
        // rounds that delivered what it forwards.
        const std::vector<iso::Round> &rounds = req->b.plan.rounds;
        auto conflict = [&](int ra, int rb) {
            for (const iso_plan_entry_t &x : rounds[(size_t)ra].entries)
                for (const iso_plan_entry_t &y : rounds[(size_t)rb].entries) {
                    const bool x_writes_what_y_touches =
                        (x.dst_buf == y.dst_buf && x.dst_slot == y.dst_slot) ||
                        (x.dst_buf == y.src_buf && x.dst_slot == y.src_slot);
                    const bool y_writes_what_x_reads = y.dst_buf == x.src_buf && y.dst_slot == x.src_slot;
                    if (x_writes_what_y_touches || y_writes_what_x_reads) return true;
                }
            return false;
        };
        hipGraph_t g = nullptr;
        ISO_HIP_TRY(hipGraphCreate(&g, 0));
        std::vector<hipGraphNode_t> nodes(req->b.launches.size());
        hipError_t e = hipSuccess;
        for (size_t i = 0; i < req->b.launches.size() && e == hipSuccess; ++i) {
            const iso::Launch &l = req->b.launches[i];
            std::vector<hipGraphNode_t> deps;
            if (enable == ISO_GRAPH_CHAIN) {
                if (i) deps.push_back(nodes[i - 1]);
            } else {
                for (size_t j = 0; j < i; ++j) {
                    const int rj = req->b.launches[j].round;
                    if (rj != l.round && conflict(rj, l.round)) deps.push_back(nodes[j]);
                }
            }
            const iso::KernelRef k = iso::select_kernel(req->b.info.vector_bytes, l);
            void *args[1] = {const_cast<void *>(k.arg)};
            hipKernelNodeParams np{};
            np.func = const_cast<void *>(k.func);
            np.gridDim = dim3(l.grid);
            np.blockDim = dim3(iso::kThreads);
            np.sharedMemBytes = l.dyn_lds;
            np.kernelParams = args;
            np.extra = nullptr;
            e = hipGraphAddKernelNode(&nodes[i], g, deps.empty() ? nullptr : deps.data(), deps.size(), &np);
        }
        if (e == hipSuccess) e = hipGraphInstantiate(&req->graph_exec, g, nullptr, nullptr, 0);
        if (e != hipSuccess) {
            (void)hipGraphDestroy(g);
            req->graph_exec = nullptr;
            g_last_hip_error = (int)e;
            (void)hipGetLastError();
            return ISO_ERR_HIP;
        }
        req->graph = g;
        req->graph_form = enable;
    }
    req->use_graph = true;
    return ISO_SUCCESS;
}

int iso_start(iso_request_t req, void *hip_stream) {
    if (!req) return ISO_ERR_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (req->use_graph) {
        ISO_HIP_TRY(hipGraphLaunch(req->graph_exec, stream));
    } else {
        for (const iso::Launch &l : req->b.launches) {
            int st = iso::enqueue(req->b.info.vector_bytes, l, stream);
            if (st != ISO_SUCCESS) return st;
        }
    }
    req->last_stream = stream;
    req->started = true;
    return ISO_SUCCESS;
}

int iso_start_range(iso_request_t req, int first, int count, void *hip_stream) {
    if (!req || first < 0 || count < 0 || (size_t)first + (size_t)count > req->b.launches.size())
        return ISO_ERR_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    for (int q = first; q < first + count; ++q) {
        int st = iso::enqueue(req->b.info.vector_bytes, req->b.launches[(size_t)q], stream);
        if (st != ISO_SUCCESS) return st;
    }
    req->last_stream = stream;
    req->started = true;
    return ISO_SUCCESS;
}

int iso_wait(iso_request_t req) {
    if (!req) return ISO_ERR_ARG;
    if (!req->started || req->b.launches.empty()) return ISO_SUCCESS;
    ISO_HIP_TRY(hipStreamSynchronize(req->last_stream));
    return ISO_SUCCESS;
}

int iso_request_info(iso_request_t req, iso_request_info_t *info) {
    if (!req || !info) return ISO_ERR_ARG;
    *info = req->b.info;
    return ISO_SUCCESS;
}

int iso_request_plan(iso_request_t req, iso_plan_t *plan) {
    return guarded([&]() -> int {
        if (!req || !plan) return ISO_ERR_ARG;
        if (req->plan_view.p.rounds.empty()) req->plan_view.p = req->b.plan;
        *plan = &req->plan_view;
        return ISO_SUCCESS;
    });
}

int iso_request_free(iso_request_t *req) {
    if (!req) return ISO_ERR_ARG;
    int st = ISO_SUCCESS;
    if (*req) {
        // the last collective may still be running: its kernels read the device table
        if ((*req)->started && !(*req)->b.launches.empty()) {
            hipError_t e = hipStreamSynchronize((*req)->last_stream);
            if (e != hipSuccess) {
                g_last_hip_error = (int)e;
                (void)hipGetLastError();
                st = ISO_ERR_HIP;
            }
        }
        if ((*req)->graph_exec) (void)hipGraphExecDestroy((*req)->graph_exec);
        if ((*req)->graph) (void)hipGraphDestroy((*req)->graph);
        if ((*req)->b.dev_table) {
            hipError_t e = hipFree((*req)->b.dev_table);
            if (e != hipSuccess) {
                g_last_hip_error = (int)e;
                (void)hipGetLastError();
                st = ISO_ERR_HIP;
            }
        }
        delete *req;
    }
    *req = nullptr;
    return st;
}

const char *iso_error_string(int status) {
    switch (status) {
        case ISO_SUCCESS: return "success";
        case ISO_ERR_ARG: return "invalid argument";
        case ISO_ERR_OVERLAP: return "buffers (or receive blocks) overlap";
        case ISO_ERR_WORKSPACE: return "workspace missing or too small";
        case ISO_ERR_HIP: return "HIP runtime error";
        case ISO_ERR_NOMEM: return "out of host memory";
        case ISO_ERR_TOO_LARGE: return "size exceeds the supported index range";
        case ISO_ERR_POINTER: return "buffer is not inside a device allocation of sufficient size";
        case ISO_ERR_SCRATCH: return "collective needs more than the library's static scratch memory holds";
        default: return "unknown status";
    }
}

int iso_last_hip_error(void) { return g_last_hip_error; }

int iso_copy_reference(const void *src, void *dst, size_t bytes, void *hip_stream) {
    if (!bytes) return ISO_SUCCESS;
    if (!src || !dst) return ISO_ERR_ARG;
    if (iso::overlap(iso::Range{(uintptr_t)src, bytes}, iso::Range{(uintptr_t)dst, bytes})) return ISO_ERR_OVERLAP;
    int st;
    if ((st = iso::check_device_range(src, bytes)) != ISO_SUCCESS) return st;
    if ((st = iso::check_device_range(dst, bytes)) != ISO_SUCCESS) return st;
    hipStream_t stream = (hipStream_t)hip_stream;
    const uint32_t l2 = iso::common_alignment_log2({(uint64_t)bytes, (uint64_t)(uintptr_t)src, (uint64_t)(uintptr_t)dst});
    const uint64_t units = bytes >> l2;
    const uint64_t blocks = (units + iso::kThreads - 1) / iso::kThreads;
    if (blocks > 0x7FFFFFFFull) return ISO_ERR_TOO_LARGE;
    const dim3 grid((uint32_t)blocks), block(iso::kThreads);
    switch (l2) {
        case 4:
            hipLaunchKernelGGL((iso::copy_kernel<iso::vec16_t>), grid, block, 0, stream,
                               (const iso::vec16_t *)src, (iso::vec16_t *)dst, units);
            break;
        case 3:
            hipLaunchKernelGGL((iso::copy_kernel<iso::vec8_t>), grid, block, 0, stream,
                               (const iso::vec8_t *)src, (iso::vec8_t *)dst, units);
            break;
        case 2:
            hipLaunchKernelGGL((iso::copy_kernel<uint32_t>), grid, block, 0, stream,
                               (const uint32_t *)src, (uint32_t *)dst, units);
            break;
        case 1:
            hipLaunchKernelGGL((iso::copy_kernel<uint16_t>), grid, block, 0, stream,
                               (const uint16_t *)src, (uint16_t *)dst, units);
            break;
        default:
            hipLaunchKernelGGL((iso::copy_kernel<uint8_t>), grid, block, 0, stream,
                               (const uint8_t *)src, (uint8_t *)dst, units);
            break;
    }
    ISO_HIP_TRY(hipGetLastError());
    return ISO_SUCCESS;
}

}  // extern "C"
