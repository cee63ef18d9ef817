// C ABI of libiso (see include/iso.h): handles, argument checks, binding of a
// schedule to device buffers, and the per-round kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "iso.h"
#include "iso_kernels.hpp"
#include "iso_plan.hpp"

namespace {

thread_local int g_last_hip_error = 0;

constexpr uint32_t kMaxUnits = 0xFFF00000u;   // flat 32-bit work index per launch

#define ISO_HIP_TRY(expr)                              \
    do {                                               \
        hipError_t err_ = (expr);                      \
        if (err_ != hipSuccess) {                      \
            g_last_hip_error = (int)err_;              \
            (void)hipGetLastError();                   \
            return ISO_ERR_HIP;                        \
        }                                              \
    } while (0)

struct Launch {
    int kind;
    uint32_t grid;
    bool lds_table;
    iso::ShiftArgs shift;
    iso::VectorArgs vec;
};

struct Range {
    uintptr_t lo;
    size_t len;
};

bool overlap(const Range &a, const Range &b) {
    if (!a.len || !b.len) return false;
    return a.lo < b.lo + b.len && b.lo < a.lo + a.len;
}

// The range must lie inside one device allocation known to the HIP runtime.
int check_device_range(const void *ptr, size_t len) {
    if (!len) return ISO_SUCCESS;
    if (!ptr) return ISO_ERR_ARG;
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    hipError_t e = hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)ptr);
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        (void)hipGetLastError();
        return ISO_ERR_POINTER;
    }
    const uintptr_t b = (uintptr_t)base, q = (uintptr_t)ptr;
    if (q < b || q - b > size || len > size - (q - b)) return ISO_ERR_POINTER;
    return ISO_SUCCESS;
}

int widest_vector(size_t m, std::initializer_list<const void *> ptrs) {
    uintptr_t bits = (uintptr_t)m;
    for (const void *p : ptrs) bits |= (uintptr_t)p;
    int v = 16;
    while (v > 1 && (bits & (uintptr_t)(v - 1))) v >>= 1;
    return v;
}

void set_grid(Launch &l, uint32_t total, uint32_t k) {
    const uint32_t n_tiles = (uint32_t)(((uint64_t)total + iso::kThreads - 1) / iso::kThreads);
    // Runs of 128 tiles (512 KiB of units) per XCD: measured best over the five workloads
    // (no runs: -5 % where the rank stride is a multiple of 4 KiB; runs of 512 tiles or more:
    // -8 % and worse, the last incomplete span leaves XCDs idle).
    uint32_t run_log2 = 7;
    while (run_log2 > 0 && (8u << run_log2) > n_tiles) --run_log2;
    const uint32_t span = 8u << run_log2;
    l.grid = (uint32_t)((((uint64_t)n_tiles + span - 1) / span) * span);
    iso::TileMap &tm = l.kind == ISO_ROUND_VECTOR ? l.vec.map : l.shift.map;
    tm.n_tiles = n_tiles;
    tm.run_log2 = run_log2;
    l.lds_table = k <= iso::kLdsEntries;
    if (l.kind == ISO_ROUND_VECTOR) {
        l.vec.total = total;
        l.vec.k = k;
    } else {
        l.shift.total = total;
        l.shift.k = k;
    }
}

template <typename V, bool LDS>
void enqueue(const Launch &l, hipStream_t stream) {
    if (l.kind == ISO_ROUND_VECTOR)
        hipLaunchKernelGGL((iso::vector_round_kernel<V, LDS>), dim3(l.grid), dim3(iso::kThreads), 0,
                           stream, l.vec);
    else
        hipLaunchKernelGGL((iso::shift_round_kernel<V, LDS>), dim3(l.grid), dim3(iso::kThreads), 0,
                           stream, l.shift);
}

template <typename V>
int launch_one(const Launch &l, hipStream_t stream) {
    if (l.lds_table)
        enqueue<V, true>(l, stream);
    else
        enqueue<V, false>(l, stream);
    ISO_HIP_TRY(hipGetLastError());
    return ISO_SUCCESS;
}

int launch_width(int vec, const Launch &l, hipStream_t stream) {
    switch (vec) {
        case 16: return launch_one<iso::vec16_t>(l, stream);
        case 8:  return launch_one<iso::vec8_t>(l, stream);
        case 4:  return launch_one<uint32_t>(l, stream);
        case 2:  return launch_one<uint16_t>(l, stream);
        default: return launch_one<uint8_t>(l, stream);
    }
}

}  // namespace

struct iso_comm_s {
    iso::Comm c;
    int64_t allgather_moves = 0;
};

struct iso_plan_s {
    iso::Plan p;
};

struct iso_request_s {
    iso_plan_s plan;
    iso_request_info_t info{};
    void *dev_table = nullptr;
    std::vector<Launch> launches;
    hipStream_t last_stream = nullptr;
    bool started = false;
    hipGraph_t graph = nullptr;          // the launches of one collective as a HIP graph
    hipGraphExec_t graph_exec = nullptr;
    bool use_graph = false;
};

namespace {

size_t work_bytes(const iso::Plan &pl, size_t m) { return (size_t)pl.work_slots * (size_t)pl.comm.p * m; }

int init_common(int op, const void *sendbuf, void *recvbuf, size_t m, void *workspace,
                size_t workspace_bytes, iso_comm_t comm, int algorithm, iso_request_t *out) {
    if (!out) return ISO_ERR_ARG;
    *out = nullptr;
    if (!comm) return ISO_ERR_ARG;
    const iso::Comm &c = comm->c;
    iso_request_s *rq = new iso_request_s();
    struct Guard {
        iso_request_s *r;
        ~Guard() {
            if (r) {
                if (r->dev_table) (void)hipFree(r->dev_table);
                delete r;
            }
        }
    } guard{rq};

    int st = iso::build_plan(c, op, algorithm, rq->plan.p);
    if (st != ISO_SUCCESS) return st;
    const iso::Plan &pl = rq->plan.p;
    const uint64_t p = (uint64_t)c.p, s = (uint64_t)c.s;
    if (m && p > (~(uint64_t)0 >> 1) / std::max<uint64_t>(1, s) / m) return ISO_ERR_TOO_LARGE;

    iso_request_info_t &inf = rq->info;
    inf.op = op; inf.algorithm = algorithm; inf.p = c.p; inf.s = c.s; inf.block_bytes = m;
    inf.entries = pl.entries();
    inf.bytes_read = inf.bytes_written = (uint64_t)inf.entries * p * m;
    inf.delivered_bytes = p * s * m;
    inf.workspace_bytes = work_bytes(pl, m);
    inf.vector_bytes = 16;

    const size_t send_len = (op == ISO_OP_ALLTOALL ? p * s : (s ? p : 0)) * m;
    const size_t recv_len = p * s * m;
    const size_t work_len = inf.workspace_bytes;
    if (send_len && !sendbuf) return ISO_ERR_ARG;
    if (recv_len && !recvbuf) return ISO_ERR_ARG;
    if (work_len && !workspace) return ISO_ERR_WORKSPACE;
    if (work_len > workspace_bytes) return ISO_ERR_WORKSPACE;
    const Range rs{(uintptr_t)sendbuf, send_len}, rr{(uintptr_t)recvbuf, recv_len},
        rw{(uintptr_t)workspace, work_len};
    if (overlap(rs, rr) || overlap(rs, rw) || overlap(rr, rw)) return ISO_ERR_OVERLAP;

    if (recv_len == 0) {          // m == 0, s == 0: nothing to move
        inf.launches = 0;
        guard.r = nullptr;
        *out = rq;
        return ISO_SUCCESS;
    }
    if ((st = check_device_range(sendbuf, send_len)) != ISO_SUCCESS) return st;
    if ((st = check_device_range(recvbuf, recv_len)) != ISO_SUCCESS) return st;
    if ((st = check_device_range(workspace, work_len)) != ISO_SUCCESS) return st;

    const int vec = work_len ? widest_vector(m, {sendbuf, recvbuf, workspace})
                             : widest_vector(m, {sendbuf, recvbuf});
    inf.vector_bytes = vec;
    const uint64_t chunks = m / (size_t)vec;
    const uint64_t units_per_entry = p * chunks;
    if (chunks > 0x7FFFFFFFu || units_per_entry > kMaxUnits) return ISO_ERR_TOO_LARGE;
    const uint32_t k_max = (uint32_t)(kMaxUnits / units_per_entry);

    // byte stride between ranks and base address per buffer kind
    const uint64_t base[3] = {(uint64_t)(uintptr_t)sendbuf, (uint64_t)(uintptr_t)recvbuf,
                              (uint64_t)(uintptr_t)workspace};
    // send and recv: the caller's rank-major [p][s][m].  Workspace: slot-major [w][p][m], so
    // that the blocks of one entry form a dense stream over the ranks whatever m is (rank-major
    // workspace rows cost 20 % at m <= 64, where a row of w blocks is touched a few sectors at a time).
    const uint64_t stride[3] = {op == ISO_OP_ALLTOALL ? s * m : m, s * m, m};
    const uint64_t slot_step[3] = {m, m, p * m};

    std::vector<iso::DevEntry> table;
    table.reserve((size_t)inf.entries);
    struct Pending { size_t first; Launch l; };
    std::vector<Pending> pending;
    for (const iso::Round &r : pl.rounds) {
        size_t done = 0;
        while (done < r.entries.size()) {
            const uint32_t k = (uint32_t)std::min<size_t>(k_max, r.entries.size() - done);
            Pending pd;
            pd.first = table.size();
            Launch &l = pd.l;
            std::memset(&l, 0, sizeof(l));
            l.kind = r.kind;
            for (uint32_t q = 0; q < k; ++q) {
                const iso_plan_entry_t &pe = r.entries[done + q];
                iso::DevEntry de{};
                de.src = base[pe.src_buf] + (uint64_t)pe.src_slot * slot_step[pe.src_buf];
                de.dst = base[pe.dst_buf] + (uint64_t)pe.dst_slot * slot_step[pe.dst_buf];
                de.src_stride = stride[pe.src_buf];
                de.dst_stride = stride[pe.dst_buf];
                de.shift = r.kind == ISO_ROUND_VECTOR ? (uint32_t)pe.neighbor : (uint32_t)pe.shift;
                table.push_back(de);
            }
            const iso::FastDiv dch = iso::make_fastdiv((uint32_t)chunks), dk = iso::make_fastdiv(k);
            if (r.kind == ISO_ROUND_VECTOR) {
                l.vec.d = c.d;
                l.vec.d_chunks = dch;
                l.vec.d_k = dk;
                for (int j = 0; j < c.d; ++j) {
                    l.vec.d_dims[j] = iso::make_fastdiv((uint32_t)c.dims[j]);
                    l.vec.inner[j] = (uint32_t)c.inner[j];
                }
            } else {
                const bool shift = r.kind == ISO_ROUND_SHIFT;
                l.shift.inner = shift ? (uint32_t)c.inner[r.dim] : 1u;
                l.shift.pj = shift ? (uint32_t)c.dims[r.dim] : 1u;
                l.shift.d_chunks = dch;
                l.shift.d_k = dk;
                l.shift.d_inner = iso::make_fastdiv(l.shift.inner);
                l.shift.d_pj = iso::make_fastdiv(l.shift.pj);
            }
            set_grid(l, (uint32_t)(units_per_entry * k), k);
            pending.push_back(pd);
            done += k;
        }
    }

    // one device table: the entries of all launches, then the [s][d] residues
    const size_t entry_bytes = table.size() * sizeof(iso::DevEntry);
    const size_t off_bytes = c.can.size() * sizeof(uint32_t);
    if (entry_bytes + off_bytes) {
        ISO_HIP_TRY(hipMalloc(&rq->dev_table, entry_bytes + off_bytes));
        if (entry_bytes)
            ISO_HIP_TRY(hipMemcpy(rq->dev_table, table.data(), entry_bytes, hipMemcpyHostToDevice));
        if (off_bytes)
            ISO_HIP_TRY(hipMemcpy((char *)rq->dev_table + entry_bytes, c.can.data(), off_bytes,
                                  hipMemcpyHostToDevice));
    }
    const iso::DevEntry *dev_entries = (const iso::DevEntry *)rq->dev_table;
    const uint32_t *dev_offsets = (const uint32_t *)((char *)rq->dev_table + entry_bytes);
    for (Pending &pd : pending) {
        if (pd.l.kind == ISO_ROUND_VECTOR) {
            pd.l.vec.entries = dev_entries + pd.first;
            pd.l.vec.offsets = dev_offsets;
        } else {
            pd.l.shift.entries = dev_entries + pd.first;
        }
        rq->launches.push_back(pd.l);
    }
    inf.launches = (int32_t)rq->launches.size();
    guard.r = nullptr;
    *out = rq;
    return ISO_SUCCESS;
}

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

}  // namespace

extern "C" {

int iso_neighborhood_create(int d, const int32_t *dims, int s, const int32_t *rel_coords,
                            iso_comm_t *comm) {
    return guarded([&]() -> int {
        if (!comm) return ISO_ERR_ARG;
        *comm = nullptr;
        iso_comm_s *h = new iso_comm_s();
        int st = iso::build_comm(d, dims, s, rel_coords, h->c);
        if (st != ISO_SUCCESS) {
            delete h;
            return st;
        }
        (void)iso::allgather_dim_order(h->c, &h->allgather_moves);
        *comm = h;
        return ISO_SUCCESS;
    });
}

int iso_neighborhood_info(iso_comm_t comm, iso_comm_info_t *info) {
    if (!comm || !info) return ISO_ERR_ARG;
    const iso::Comm &c = comm->c;
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
        *bytes = work_bytes(pl, m);
        return ISO_SUCCESS;
    });
}

int iso_neighbor_alltoall_init(const void *sendbuf, void *recvbuf, size_t m, void *workspace,
                               size_t workspace_bytes, iso_comm_t comm, int algorithm,
                               iso_request_t *req) {
    return guarded([&]() -> int {
        return init_common(ISO_OP_ALLTOALL, sendbuf, recvbuf, m, workspace, workspace_bytes, comm,
                           algorithm, req);
    });
}

int iso_neighbor_allgather_init(const void *sendbuf, void *recvbuf, size_t m, void *workspace,
                                size_t workspace_bytes, iso_comm_t comm, int algorithm,
                                iso_request_t *req) {
    return guarded([&]() -> int {
        return init_common(ISO_OP_ALLGATHER, sendbuf, recvbuf, m, workspace, workspace_bytes, comm,
                           algorithm, req);
    });
}

int iso_request_set_graph(iso_request_t req, int enable) {
    if (!req) return ISO_ERR_ARG;
    if (!enable || req->launches.empty()) {
        req->use_graph = false;
        return ISO_SUCCESS;
    }
    if (!req->graph_exec) {
        // record the launch sequence once on a private stream, then replay it
        hipStream_t cs = nullptr;
        ISO_HIP_TRY(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
        hipError_t e = hipStreamBeginCapture(cs, hipStreamCaptureModeRelaxed);
        int st = ISO_SUCCESS;
        if (e == hipSuccess) {
            for (const Launch &l : req->launches)
                if ((st = launch_width(req->info.vector_bytes, l, cs)) != ISO_SUCCESS) break;
            hipGraph_t g = nullptr;
            e = hipStreamEndCapture(cs, &g);
            if (e == hipSuccess && st == ISO_SUCCESS) {
                e = hipGraphInstantiate(&req->graph_exec, g, nullptr, nullptr, 0);
                req->graph = g;
            } else if (g) {
                (void)hipGraphDestroy(g);
            }
        }
        (void)hipStreamDestroy(cs);
        if (st != ISO_SUCCESS) return st;
        if (e != hipSuccess) {
            if (req->graph) (void)hipGraphDestroy(req->graph);
            req->graph = nullptr;
            req->graph_exec = nullptr;
            g_last_hip_error = (int)e;
            (void)hipGetLastError();
            return ISO_ERR_HIP;
        }
    }
    req->use_graph = true;
    return ISO_SUCCESS;
}

int iso_start(iso_request_t req, void *hip_stream) {
    if (!req) return ISO_ERR_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (req->use_graph) {
        ISO_HIP_TRY(hipGraphLaunch(req->graph_exec, stream));
        req->last_stream = stream;
        req->started = true;
        return ISO_SUCCESS;
    }
    for (const Launch &l : req->launches) {
        int st = launch_width(req->info.vector_bytes, l, stream);
        if (st != ISO_SUCCESS) return st;
    }
    req->last_stream = stream;
    req->started = true;
    return ISO_SUCCESS;
}

int iso_start_range(iso_request_t req, int first, int count, void *hip_stream) {
    if (!req || first < 0 || count < 0 || (size_t)first + (size_t)count > req->launches.size())
        return ISO_ERR_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    for (int q = first; q < first + count; ++q) {
        int st = launch_width(req->info.vector_bytes, req->launches[(size_t)q], stream);
        if (st != ISO_SUCCESS) return st;
    }
    req->last_stream = stream;
    req->started = true;
    return ISO_SUCCESS;
}

int iso_wait(iso_request_t req) {
    if (!req) return ISO_ERR_ARG;
    if (!req->started || req->launches.empty()) return ISO_SUCCESS;
    ISO_HIP_TRY(hipStreamSynchronize(req->last_stream));
    return ISO_SUCCESS;
}

int iso_request_info(iso_request_t req, iso_request_info_t *info) {
    if (!req || !info) return ISO_ERR_ARG;
    *info = req->info;
    return ISO_SUCCESS;
}

int iso_request_plan(iso_request_t req, iso_plan_t *plan) {
    if (!req || !plan) return ISO_ERR_ARG;
    *plan = &req->plan;
    return ISO_SUCCESS;
}

int iso_request_free(iso_request_t *req) {
    if (!req) return ISO_ERR_ARG;
    int st = ISO_SUCCESS;
    if (*req) {
        if ((*req)->graph_exec) (void)hipGraphExecDestroy((*req)->graph_exec);
        if ((*req)->graph) (void)hipGraphDestroy((*req)->graph);
        if ((*req)->dev_table) {
            hipError_t e = hipFree((*req)->dev_table);
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
        case ISO_ERR_OVERLAP: return "send, receive and workspace buffers overlap";
        case ISO_ERR_WORKSPACE: return "workspace missing or too small";
        case ISO_ERR_HIP: return "HIP runtime error";
        case ISO_ERR_NOMEM: return "out of host memory";
        case ISO_ERR_TOO_LARGE: return "size exceeds the supported index range";
        case ISO_ERR_POINTER: return "buffer is not inside a device allocation of sufficient size";
        default: return "unknown status";
    }
}

int iso_last_hip_error(void) { return g_last_hip_error; }

int iso_copy_reference(const void *src, void *dst, size_t bytes, void *hip_stream) {
    if (!bytes) return ISO_SUCCESS;
    if (!src || !dst) return ISO_ERR_ARG;
    if (overlap(Range{(uintptr_t)src, bytes}, Range{(uintptr_t)dst, bytes})) return ISO_ERR_OVERLAP;
    int st;
    if ((st = check_device_range(src, bytes)) != ISO_SUCCESS) return st;
    if ((st = check_device_range(dst, bytes)) != ISO_SUCCESS) return st;
    hipStream_t stream = (hipStream_t)hip_stream;
    const int vec = widest_vector(bytes, {src, dst});
    const uint64_t units = bytes / (size_t)vec;
    const uint64_t blocks = (units + iso::kThreads - 1) / iso::kThreads;
    if (blocks > 0x7FFFFFFFull) return ISO_ERR_TOO_LARGE;
    const dim3 grid((uint32_t)blocks), block(iso::kThreads);
    switch (vec) {
        case 16:
            hipLaunchKernelGGL((iso::copy_kernel<iso::vec16_t>), grid, block, 0, stream,
                               (const iso::vec16_t *)src, (iso::vec16_t *)dst, units);
            break;
        case 8:
            hipLaunchKernelGGL((iso::copy_kernel<iso::vec8_t>), grid, block, 0, stream,
                               (const iso::vec8_t *)src, (iso::vec8_t *)dst, units);
            break;
        case 4:
            hipLaunchKernelGGL((iso::copy_kernel<uint32_t>), grid, block, 0, stream,
                               (const uint32_t *)src, (uint32_t *)dst, units);
            break;
        case 2:
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
