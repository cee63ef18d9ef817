// Binding of a schedule to device buffers: turns a plan plus a block layout
// (sizes and displacements of the s blocks in a rank's send and receive rows)
// into the device table of block index maps and the list of kernel launches.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <initializer_list>
#include <numeric>
#include <vector>

#include "iso.h"
#include "iso_kernels.hpp"
#include "iso_plan.hpp"

namespace iso {

extern thread_local int g_last_hip_error;

constexpr uint32_t kMaxUnits = 0xFFF00000u;   // flat 32-bit work index per launch

#define ISO_HIP_TRY(expr)                              \
    do {                                               \
        hipError_t err_ = (expr);                      \
        if (err_ != hipSuccess) {                      \
            iso::g_last_hip_error = (int)err_;         \
            (void)hipGetLastError();                   \
            return ISO_ERR_HIP;                        \
        }                                              \
    } while (0)

enum LaunchKernel { kShiftKernel = 0, kVectorKernel = 1, kBlockKernel = 2, kMeshShiftKernel = 3, kDeliverKernel = 4, kStagedRoundKernel = 5 };

struct Launch {
    int kernel;            // LaunchKernel
    uint32_t grid;
    bool lds_table;
    bool mesh;
    bool stream_loads;     // every source block is read exactly once in this launch: non-temporal loads
    bool tail;             // regular kernels: the last unit of a block overlaps the one before it
    bool uniform_waves;    // shift kernel, 16-byte units, blocks a multiple of 64 units: one block per wavefront
    bool block_groups;     // block kernel: ranks taken in groups of kBlockGroup
    int round;             // the plan's round this launch belongs to (a large round is split over several launches)
    uint32_t dyn_lds;      // bytes of dynamic LDS (the kernels of the staged schedule: their tile)

    ShiftArgs shift;
    VectorArgs vec;
    BlockArgs block;
    MeshArgs mesh_shift;
    DeliverArgs deliver;
    StagedRoundArgs staged;
    uint32_t tile_units;   // the staged schedule's kernels: kTileUnits or kSmallTileUnits
};

// Sizes and displacements (bytes) of the s blocks inside one rank's send and
// receive rows, and the distance between consecutive ranks' rows.
struct Layout {
    std::vector<uint64_t> size, send_displ, recv_displ;
    uint64_t send_extent = 0, recv_extent = 0;
    uint64_t send_span = 0, recv_span = 0;    // first to last byte of one rank's blocks
    bool slot_major = false;                  // one plane per neighbour: consecutive ranks' blocks i are
                                              // size[i] bytes apart (regular blocks: [s][p][m]); the
                                              // extents then only describe the allgather's send rows
};

struct Range {
    uintptr_t lo;
    size_t len;
};

inline bool overlap(const Range &a, const Range &b) {
    if (!a.len || !b.len) return false;
    return a.lo < b.lo + b.len && b.lo < a.lo + a.len;
}

// The range must lie inside one device allocation known to the HIP runtime.
inline int check_device_range(const void *ptr, size_t len) {
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

// log2 of the widest power of two (<= 16) that divides all the values: the access width of the
// plain reference copy, which keeps naturally aligned accesses
inline uint32_t common_alignment_log2(std::initializer_list<uint64_t> values) {
    uint64_t bits = 0;
    for (uint64_t v : values) bits |= v;
    uint32_t l = 4;
    while (l > 0 && (bits & ((uint64_t(1) << l) - 1))) --l;
    return l;
}

// log2 of the unit width for a block of `size` >= 1 bytes: the largest power of two that is
// at most 16 and at most the size (the last unit of a block overlaps its predecessor when the
// width does not divide the size; addresses need no alignment)
inline uint32_t unit_log2_of(uint64_t size) {
    uint32_t l = 4;
    while (l > 0 && (uint64_t(1) << l) > size) --l;
    return l;
}

inline uint64_t align16(uint64_t x) { return (x + 15) & ~uint64_t(15); }

// Slot-major workspace: slot w holds one block per rank, p * size_w bytes, slots
// back to back (each start rounded up to 16 bytes).  Dense streams per entry
// whatever the block size is.
struct WorkLayout {
    std::vector<uint64_t> size, offset;
    uint64_t bytes = 0;
};

inline WorkLayout work_layout(const Plan &pl, const Layout &lay) {
    WorkLayout w;
    w.size.assign((size_t)pl.work_slots, 0);
    w.offset.assign((size_t)pl.work_slots, 0);
    const uint64_t uniform = lay.size.empty() ? 0 : lay.size[0];
    for (const Round &r : pl.rounds)
        for (const iso_plan_entry_t &e : r.entries)
            if (e.dst_buf == ISO_BUF_WORK) {
                const uint64_t sz = (pl.op == ISO_OP_ALLTOALL && e.neighbor >= 0) ? lay.size[(size_t)e.neighbor]
                                                                                  : uniform;
                w.size[(size_t)e.dst_slot] = std::max(w.size[(size_t)e.dst_slot], sz);
            }
    for (int q = 0; q < pl.work_slots; ++q) {
        w.offset[(size_t)q] = w.bytes;
        w.bytes += align16((uint64_t)pl.comm.p * w.size[(size_t)q]);
    }
    return w;
}

// Blocks that sit at a rank stride that is a multiple of 4 KiB and cover only part of the offsets
// modulo 4 KiB (config 3: 1 KiB blocks in 12 KiB rows) use a fraction of what the address bits
// below 4 KiB select in the memory system, whichever ranks are in flight.  How the eight XCDs'
// streams lie to each other then matters: measured on plain strided copies of 256 B - 2 KiB
// pieces, strides that are multiples of 4 KiB run 4 - 26 % faster when every XCD sweeps its own
// contiguous eighth of the tiles than with interleaved runs (multiples of 8 KiB gain most), all
// other strides are indifferent to it (within 1 %) and dense or page-covering launches prefer runs.
// `sides`: per entry its (address, stride, block size) on the source and on the destination side.
struct Side {
    uint64_t addr, stride, size;
};

inline bool page_resonant(const std::vector<Side> &sides) {
    bool marked[256] = {};                     // 16-byte granules of a 4 KiB page
    bool any = false;
    for (const Side &sd : sides) {
        if (!sd.size || !sd.stride || (sd.stride & 4095u)) continue;
        any = true;
        const uint64_t lo = (sd.addr & 4095u) >> 4, n = std::min<uint64_t>(256, (sd.size + (sd.addr & 15u) + 15) >> 4);
        for (uint64_t q = 0; q < n; ++q) marked[(lo + q) & 255u] = true;
    }
    if (!any) return false;
    for (bool b : marked)
        if (!b) return true;
    return false;
}

inline void set_grid(Launch &l, uint32_t total, uint32_t k, bool eighths) {
    const uint32_t n_tiles = (uint32_t)(((uint64_t)total + kThreads - 1) / kThreads);
    // Runs of 128 tiles (512 KiB of units) per XCD: measured best over the five workloads
    // (no runs: -5 % where the rank stride is a multiple of 4 KiB; runs of 512 tiles or more:
    // -8 % and worse, the last incomplete span leaves XCDs idle).
    uint32_t run_log2 = 7;
    // (the staged schedule's kernels: a tile is 32 KiB and there are few of them; with runs of 128 a grid
    // padded to whole spans had up to 18 % workgroups without a tile, which cost 7 % at 16-byte blocks; runs
    // of 4 ... 32 tiles measure alike)
    if (l.kernel == kStagedRoundKernel || l.kernel == kDeliverKernel) run_log2 = 3;
    while (run_log2 > 0 && (8u << run_log2) > n_tiles) --run_log2;
    const uint32_t span = 8u << run_log2;
    l.grid = (uint32_t)((((uint64_t)n_tiles + span - 1) / span) * span);
    const uint32_t per_xcd = (n_tiles + 7) / 8;
    if (eighths && n_tiles >= 64) {            // one contiguous eighth per XCD (balanced for any tile count)
        run_log2 = kEighths;
        l.grid = per_xcd * 8;
    }
    TileMap &tm = l.kernel == kVectorKernel  ? l.vec.map
                  : l.kernel == kStagedRoundKernel ? l.staged.map
                  : l.kernel == kDeliverKernel ? l.deliver.map
                  : l.kernel == kBlockKernel ? l.block.map
                  : l.kernel == kMeshShiftKernel ? l.mesh_shift.map
                                                 : l.shift.map;
    tm.n_tiles = n_tiles;
    tm.run_log2 = run_log2;
    tm.per_xcd = per_xcd;
    l.lds_table = k <= kLdsEntries;
    if (l.kernel == kStagedRoundKernel || l.kernel == kDeliverKernel) {
        // one tile per workgroup: `total` counts tiles * kThreads here
    } else if (l.kernel == kVectorKernel) {
        l.vec.total = total;
        l.vec.k = k;
    } else if (l.kernel == kBlockKernel) {
        l.block.total = total;
        l.block.k = k;
    } else if (l.kernel == kMeshShiftKernel) {
        l.mesh_shift.total = total;
        l.mesh_shift.k = k;
    } else {
        l.shift.total = total;
        l.shift.k = k;
    }
}

// Which instantiation runs a launch, and the argument struct it takes: resolved once per launch,
// used both for plain launches and for the kernel nodes of a request's graph.
struct KernelRef {
    const void *func;
    const void *arg;
};

// Streaming loads exist for the shift kernel at the 16-byte width only (narrower
// units are the slow path anyway).
template <typename V, bool LDS, bool TAIL>
KernelRef select_regular(const Launch &l) {
    if (l.kernel == kVectorKernel) return {(const void *)&vector_round_kernel<V, LDS, TAIL>, &l.vec};
    if (l.kernel == kMeshShiftKernel) {
        if constexpr (sizeof(V) == 16) {
            if (l.stream_loads) return {(const void *)&mesh_shift_round_kernel<V, LDS, true, TAIL>, &l.mesh_shift};
        }
        return {(const void *)&mesh_shift_round_kernel<V, LDS, false, TAIL>, &l.mesh_shift};
    }
    if constexpr (sizeof(V) == 16) {
        if (l.uniform_waves) {
            if (l.shift.group) {
                if (l.stream_loads) return {(const void *)&shift_round_uniform_kernel<true, true>, &l.shift};
                return {(const void *)&shift_round_uniform_kernel<false, true>, &l.shift};
            }
            if (l.stream_loads) return {(const void *)&shift_round_uniform_kernel<true>, &l.shift};
            return {(const void *)&shift_round_uniform_kernel<false>, &l.shift};
        }
        if (l.shift.group) {
            if (l.stream_loads) return {(const void *)&shift_round_kernel<V, LDS, true, TAIL, true>, &l.shift};
            return {(const void *)&shift_round_kernel<V, LDS, false, TAIL, true>, &l.shift};
        }
        if (l.stream_loads) return {(const void *)&shift_round_kernel<V, LDS, true, TAIL>, &l.shift};
    }
    return {(const void *)&shift_round_kernel<V, LDS, false, TAIL>, &l.shift};
}

template <typename V>
KernelRef select_width(const Launch &l) {
    if constexpr (sizeof(V) > 1) {
        if (l.tail) {                     // the unit width does not divide the block size
            if (l.lds_table) return select_regular<V, true, true>(l);
            return select_regular<V, false, true>(l);
        }
    }
    if (l.lds_table) return select_regular<V, true, false>(l);
    return select_regular<V, false, false>(l);
}

template <bool LDS, bool MESH>
KernelRef select_block(const Launch &l) {
    if (l.block_groups) {
        if (l.stream_loads) return {(const void *)&block_round_kernel<LDS, MESH, true, true>, &l.block};
        return {(const void *)&block_round_kernel<LDS, MESH, false, true>, &l.block};
    }
    if (l.stream_loads) return {(const void *)&block_round_kernel<LDS, MESH, true>, &l.block};
    return {(const void *)&block_round_kernel<LDS, MESH, false>, &l.block};
}

inline KernelRef select_kernel(int vector_bytes, const Launch &l) {
    if (l.kernel == kStagedRoundKernel) {                 // blocks of whole 16-byte units only
        if (l.tile_units == kSmallTileUnits) {
            if (l.stream_loads) return {(const void *)&staged_round_kernel<vec16_t, true, kSmallTileUnits / kThreads>, &l.staged};
            return {(const void *)&staged_round_kernel<vec16_t, false, kSmallTileUnits / kThreads>, &l.staged};
        }
        if (l.stream_loads) return {(const void *)&staged_round_kernel<vec16_t, true, kTileUnits / kThreads>, &l.staged};
        return {(const void *)&staged_round_kernel<vec16_t, false, kTileUnits / kThreads>, &l.staged};
    }
    if (l.kernel == kDeliverKernel) {
        if (l.tile_units == kSmallTileUnits) {
            if (l.stream_loads) return {(const void *)&deliver_kernel<vec16_t, true, kSmallTileUnits / kThreads>, &l.deliver};
            return {(const void *)&deliver_kernel<vec16_t, false, kSmallTileUnits / kThreads>, &l.deliver};
        }
        if (l.stream_loads) return {(const void *)&deliver_kernel<vec16_t, true, kTileUnits / kThreads>, &l.deliver};
        return {(const void *)&deliver_kernel<vec16_t, false, kTileUnits / kThreads>, &l.deliver};
    }
    if (l.kernel == kBlockKernel) {
        if (l.mesh) return l.lds_table ? select_block<true, true>(l) : select_block<false, true>(l);
        return l.lds_table ? select_block<true, false>(l) : select_block<false, false>(l);
    }
    switch (vector_bytes) {
        case 16: return select_width<vec16_t>(l);
        case 8:  return select_width<vec8_t>(l);
        case 4:  return select_width<uint32_t>(l);
        case 2:  return select_width<uint16_t>(l);
        default: return select_width<uint8_t>(l);
    }
}

inline int enqueue(int vector_bytes, const Launch &l, hipStream_t stream) {
    const KernelRef k = select_kernel(vector_bytes, l);
    void *args[1] = {const_cast<void *>(k.arg)};
    ISO_HIP_TRY(hipLaunchKernel(k.func, dim3(l.grid), dim3(kThreads), args, l.dyn_lds, stream));
    return ISO_SUCCESS;
}

struct BoundRequest {
    Plan plan;
    iso_request_info_t info{};
    void *dev_table = nullptr;         // owned (hipMalloc) unless the request was bound to a StaticArena
    std::vector<Launch> launches;
};

// Device memory that the library already holds, for binding a schedule without allocating:
// the table of block index maps goes to `table` (written by table_store_kernel launches on
// `stream`, ordered before the rounds that read it), and the caller of bind_request passes the
// rest of the arena as the workspace.  Nothing is allocated, copied or freed.
struct StaticArena {
    unsigned char *table;              // device address, 16-byte aligned
    size_t table_bytes;
    hipStream_t stream;
};

inline int store_table(const StaticArena &arena, size_t at, const void *host, size_t bytes) {
    // `at` and `bytes` are multiples of 4: every part of the table is an array of 32-bit words or of DevEntry
    const uint32_t *w = (const uint32_t *)host;
    size_t words = bytes / 4, done = 0;
    while (done < words) {
        TableChunk ch;
        ch.dst = (uint32_t *)(arena.table + at) + done;
        ch.n = (uint32_t)std::min<size_t>(kStoreWords, words - done);
        ch.reserved = 0;
        std::memcpy(ch.words, w + done, (size_t)ch.n * 4);
        hipLaunchKernelGGL(table_store_kernel, dim3((ch.n + kThreads - 1) / kThreads), dim3(kThreads), 0,
                           arena.stream, ch);
        ISO_HIP_TRY(hipGetLastError());
        done += ch.n;
    }
    return ISO_SUCCESS;
}

// One entry of a launch on the host: the device entry, the block's size, and for the staged schedule's last
// launch the dimension the entry moves along and the receive block it writes.
struct HostEntry {
    DevEntry de;
    uint64_t size;
    int dim, dst_slot;
};

// Mesh shift launches of equal blocks: one bit per tile of kThreads units, set where every rank of the tile has
// a source for every entry of the launch.  Coordinates at which every entry finds its source: r_l - c_l in
// [0, p_l) for all masked dimensions l of all entries.  A tile is interior if its ranks share all coordinates
// but the last and lie inside these bounds (conservative: a tile that crosses into the next row of the last
// dimension counts as not interior).
inline std::vector<uint32_t> mesh_interior_tiles(const Comm &c, bool slot_major, const HostEntry *ents, uint32_t k,
                                                 uint64_t total, uint64_t chunks, uint64_t p) {
    std::vector<int64_t> in_lo((size_t)c.d, 0), in_hi((size_t)c.d, 0);
    bool has_interior = true;
    for (int j = 0; j < c.d; ++j) {
        int64_t lo = 0, hi = c.dims[j];
        for (uint32_t q = 0; q < k; ++q) {
            const DevEntry &de = ents[q].de;
            if (!(((de.meta >> 8) >> j) & 1u)) continue;
            const int64_t cl = c.c((int)de.ref, j);
            lo = std::max<int64_t>(lo, cl);
            hi = std::min<int64_t>(hi, (int64_t)c.dims[j] + cl);
        }
        if (lo >= hi) has_interior = false;
        in_lo[(size_t)j] = lo;
        in_hi[(size_t)j] = hi;
    }
    const uint64_t n_tiles = (total + kThreads - 1) / kThreads;
    std::vector<uint32_t> bits((size_t)((n_tiles + 31) / 32), 0u);
    for (uint64_t tl = 0; has_interior && tl < n_tiles; ++tl) {
        const uint64_t u0 = tl * kThreads, u1 = std::min<uint64_t>(u0 + kThreads, total) - 1;
        const uint64_t t0 = u0 / chunks, t1 = u1 / chunks;
        uint64_t R0, R1;
        if (slot_major) {                      // (entry, rank, chunk): one entry per interior tile
            if (t0 / p != t1 / p) continue;
            R0 = t0 % p;
            R1 = t1 % p;
        } else {                               // (rank, entry, chunk)
            R0 = t0 / k;
            R1 = t1 / k;
        }
        uint64_t rem = R0;
        bool inside = true;
        for (int j = c.d - 1; j >= 0 && inside; --j) {
            const int64_t r = (int64_t)(rem % (uint64_t)c.dims[j]);
            rem /= (uint64_t)c.dims[j];
            const int64_t last = j == c.d - 1 ? r + (int64_t)(R1 - R0) : r;
            inside = r >= in_lo[(size_t)j] && last < in_hi[(size_t)j];
        }
        if (inside) bits[(size_t)(tl >> 5)] |= 1u << (tl & 31);
    }
    return bits;
}

// The record of one entry of the staged schedule's last launch.
inline DeliverEntry make_deliver_entry(const Comm &c, const HostEntry &he) {
    DeliverEntry x{};
    x.src = he.de.src;
    x.src_stride = he.de.src_stride;
    x.slot = (uint32_t)he.dst_slot;
    const uint32_t inner = he.dim < 0 ? 1u : (uint32_t)c.inner[(size_t)he.dim];
    x.pj = he.dim < 0 ? 1u : (uint32_t)c.dims[(size_t)he.dim];
    x.shift = he.dim < 0 ? 0u : he.de.shift;
    x.back = x.shift * inner;
    x.wrap = x.pj * inner;
    x.d_inner = make_fastdiv(inner);
    x.d_pj = make_fastdiv(x.pj);
    return x;
}

// Binds a schedule (`rq.plan`) to buffers: checks the buffers, builds the device table and the launch
// list.  bind_request below runs the steps in order.
// With `arena` the table is placed there instead of in an allocation of its own, and the workspace is
// taken to be the library's own memory (no look-up of its allocation); ISO_ERR_SCRATCH if either does not fit.
class Binder {
public:
    Binder(BoundRequest &request, const Comm &comm, const Layout &layout, const void *send, void *recv, void *work,
           size_t work_bytes, const StaticArena *static_arena)
        : rq(request), c(comm), lay(layout), sendbuf(send), recvbuf(recv), workspace(work),
          workspace_bytes(work_bytes), arena(static_arena), pl(request.plan), op(request.plan.op),
          p((uint64_t)comm.p), s((size_t)comm.s), inf(request.info), wl(work_layout(request.plan, layout)) {}

    int run() {
        int st = describe_and_check();
        if (st != ISO_SUCCESS || inf.delivered_bytes == 0) return st;       // nothing to move: no launches
        rounds_as_launched();
        if ((st = host_entries()) != ISO_SUCCESS) return st;
        for (size_t ri = 0; ri < bound_rounds.size(); ++ri)
            for (size_t done = 0; done < rounds[ri].size();)
                if ((st = next_launch(ri, done)) != ISO_SUCCESS) return st;
        return upload();
    }

private:
    BoundRequest &rq;
    const Comm &c;
    const Layout &lay;
    const void *sendbuf;
    void *recvbuf, *workspace;
    size_t workspace_bytes;
    const StaticArena *arena;
    const Plan &pl;
    const int op;
    const uint64_t p;
    const size_t s;
    iso_request_info_t &inf;
    const WorkLayout wl;

    std::vector<Round> bound_rounds;              // the plan's rounds as launched
    std::vector<int> round_of;                    // their index in the plan
    std::vector<std::vector<HostEntry>> rounds;   // their entries that move something
    bool uniform = true;                          // all these entries have `size0` bytes
    uint64_t size0 = 0;
    uint32_t min_log2 = 4;                        // the narrowest unit width among them

    std::vector<DevEntry> table;
    std::vector<uint32_t> prefixes;               // what launches read besides their entries (see upload)
    struct Pending { size_t first_entry, first_prefix; Launch l; };
    std::vector<Pending> pending;

    uint64_t entry_size(const iso_plan_entry_t &e) const {
        if (op == ISO_OP_ALLTOALL) return lay.size[(size_t)e.neighbor];
        return s ? lay.size[0] : 0;
    }

    // bytes from the buffer's start to the end of the last block
    size_t buffer_len(const std::vector<uint64_t> &displ, uint64_t extent, uint64_t span, bool planes) const {
        if (!inf.delivered_bytes || !p) return 0;
        if (!planes) return (size_t)((p - 1) * extent + span);
        uint64_t end = 0;
        for (size_t i = 0; i < s; ++i)
            if (lay.size[i]) end = std::max(end, displ[i] + p * lay.size[i]);
        return (size_t)end;
    }

    // address of rank 0's block and byte stride between ranks, per (buffer, slot)
    void place(int buf, int slot, uint64_t &addr, uint64_t &stride) const {
        if (buf == ISO_BUF_SEND) {
            addr = (uint64_t)(uintptr_t)sendbuf + (op == ISO_OP_ALLTOALL ? lay.send_displ[(size_t)slot] : lay.send_displ[0]);
            stride = (lay.slot_major && op == ISO_OP_ALLTOALL) ? lay.size[(size_t)slot] : lay.send_extent;
        } else if (buf == ISO_BUF_RECV) {
            addr = (uint64_t)(uintptr_t)recvbuf + lay.recv_displ[(size_t)slot];
            stride = lay.slot_major ? lay.size[(size_t)slot] : lay.recv_extent;
        } else {
            addr = (uint64_t)(uintptr_t)workspace + wl.offset[(size_t)slot];
            stride = wl.size[(size_t)slot];
        }
    }

    // Fills the request's description and checks sizes, pointers and overlaps.
    int describe_and_check() {
        inf.op = op; inf.algorithm = pl.algorithm; inf.p = c.p; inf.s = c.s;
        inf.entries = pl.entries();
        inf.vector_bytes = 16;
        inf.block_bytes = 0;
        inf.delivered_bytes = 0;
        inf.launches = 0;
        for (size_t i = 0; i < s; ++i) {
            inf.block_bytes = std::max<uint64_t>(inf.block_bytes, lay.size[i]);
            inf.delivered_bytes += p * lay.size[i];
        }
        const uint64_t limit = ~uint64_t(0) >> 2;
        if (p && (lay.send_extent > limit / p || lay.recv_extent > limit / p)) return ISO_ERR_TOO_LARGE;

        inf.workspace_bytes = wl.bytes;
        inf.bytes_read = 0;
        for (const Round &r : pl.rounds)
            for (const iso_plan_entry_t &e : r.entries) inf.bytes_read += p * entry_size(e);
        inf.bytes_written = inf.bytes_read;

        const size_t send_len = buffer_len(lay.send_displ, lay.send_extent, lay.send_span,
                                           lay.slot_major && op == ISO_OP_ALLTOALL);
        const size_t recv_len = buffer_len(lay.recv_displ, lay.recv_extent, lay.recv_span, lay.slot_major);
        const size_t work_len = inf.delivered_bytes ? (size_t)wl.bytes : 0;
        if (send_len && !sendbuf) return ISO_ERR_ARG;
        if (recv_len && !recvbuf) return ISO_ERR_ARG;
        if (work_len && !workspace) return ISO_ERR_WORKSPACE;
        if (work_len > workspace_bytes) return arena ? ISO_ERR_SCRATCH : ISO_ERR_WORKSPACE;
        const Range rs{(uintptr_t)sendbuf, send_len}, rr{(uintptr_t)recvbuf, recv_len},
            rw{(uintptr_t)workspace, work_len};
        if (overlap(rs, rr) || overlap(rs, rw) || overlap(rr, rw)) return ISO_ERR_OVERLAP;
        if (inf.delivered_bytes == 0) return ISO_SUCCESS;       // all blocks empty, or no neighbours
        int st;
        if ((st = check_device_range(sendbuf, send_len)) != ISO_SUCCESS) return st;
        if ((st = check_device_range(recvbuf, recv_len)) != ISO_SUCCESS) return st;
        if (!arena && (st = check_device_range(workspace, work_len)) != ISO_SUCCESS) return st;
        return ISO_SUCCESS;
    }

    // The last launch of the staged schedule has a kernel of its own for equal blocks in dense
    // [p][s][m] receive rows; anywhere else it runs as one launch per dimension on the general kernels.
    void rounds_as_launched() {
        for (size_t ri = 0; ri < pl.rounds.size(); ++ri) {
            const Round &r = pl.rounds[ri];
            bool whole = r.kind != ISO_ROUND_DELIVER;
            if (!whole) {
                const uint64_t m0 = s ? lay.size[0] : 0;              // blocks of whole 16-byte units
                whole = m0 > 0 && m0 % 16 == 0 && !lay.slot_major && !c.mesh && r.entries.size() == s &&
                        s <= kLdsEntries && s * (m0 / 16) <= kTileUnits && lay.recv_extent == s * m0;
                for (size_t i = 0; whole && i < s; ++i)
                    whole = lay.size[i] == m0 && lay.recv_displ[i] == i * m0 && r.entries[i].dst_slot == (int)i;
            }
            if (whole) {
                bound_rounds.push_back(r);
                round_of.push_back((int)ri);
                continue;
            }
            for (int j = -1; j < c.d; ++j) {
                Round part;
                part.kind = j < 0 ? ISO_ROUND_SELF : ISO_ROUND_SHIFT;
                part.dim = j;
                for (const iso_plan_entry_t &pe : r.entries)
                    if (pe.dim == j) part.entries.push_back(pe);
                if (part.entries.empty()) continue;
                bound_rounds.push_back(std::move(part));
                round_of.push_back((int)ri);
            }
        }
    }

    // All entries with their addresses, strides and their own unit width.
    int host_entries() {
        rounds.assign(bound_rounds.size(), {});
        bool first = true;
        for (size_t ri = 0; ri < bound_rounds.size(); ++ri) {
            const Round &r = bound_rounds[ri];
            for (const iso_plan_entry_t &pe : r.entries) {
                HostEntry he{};
                he.size = entry_size(pe);
                he.dim = pe.dim;
                he.dst_slot = pe.dst_slot;
                if (he.size == 0) continue;                       // empty blocks make no move
                uint64_t src_stride = 0, dst_stride = 0;
                place(pe.src_buf, pe.src_slot, he.de.src, src_stride);
                place(pe.dst_buf, pe.dst_slot, he.de.dst, dst_stride);
                // the kernels multiply a rank by a 32-bit stride
                if ((src_stride | dst_stride) >> 32) return ISO_ERR_TOO_LARGE;
                he.de.src_stride = (uint32_t)src_stride;
                he.de.dst_stride = (uint32_t)dst_stride;
                he.de.shift = r.kind == ISO_ROUND_VECTOR ? (uint32_t)pe.neighbor : (uint32_t)pe.shift;
                const uint32_t l2 = unit_log2_of(he.size);
                const uint64_t width = uint64_t(1) << l2;
                const uint64_t units = (he.size + width - 1) >> l2;
                if (units > 0x7FFFFFFFu) return ISO_ERR_TOO_LARGE;
                he.de.units = (uint32_t)units;
                he.de.last_offset = he.size - width;
                he.de.ref = (uint32_t)pe.ref;
                // mesh: the non-periodic dimensions routed so far in which C^ref is non-zero
                uint32_t mask = 0;
                if (c.mesh && r.kind != ISO_ROUND_SELF)
                    for (int t = 0; t < c.d; ++t) {
                        const int l = pl.dim_order[(size_t)t];
                        if (!c.periodic[(size_t)l] && c.c(pe.ref, l) != 0) mask |= 1u << l;
                        if (r.kind == ISO_ROUND_SHIFT && l == r.dim) break;
                    }
                he.de.meta = l2 | (mask << 8);
                if (first) { size0 = he.size; first = false; }
                uniform = uniform && he.size == size0;
                min_log2 = std::min(min_log2, l2);
                rounds[ri].push_back(he);
            }
        }
        inf.vector_bytes = 1 << min_log2;
        return ISO_SUCCESS;
    }

    // The next launch of round `ri`: as many of its entries from `done` on as one launch takes.
    int next_launch(size_t ri, size_t &done) {
        const Round &r = bound_rounds[ri];
        const std::vector<HostEntry> &ents = rounds[ri];
        Pending pd{};
        pd.first_entry = table.size();
        pd.first_prefix = prefixes.size();
        Launch &l = pd.l;
        std::memset(&l, 0, sizeof(l));
        l.round = round_of[ri];
        uint32_t k = 0;
        uint64_t total = 0;
        // staged schedule, last launch: whole receive rows through LDS (left as one round only for
        // regular [p][s][m] rows, see rounds_as_launched)
        const bool deliver = r.kind == ISO_ROUND_DELIVER;
        // staged schedule, the rounds: all destinations are planes of the workspace; small equal blocks
        // are re-tiled through LDS (any round of that schedule whose blocks of one rank fit a tile)
        const uint64_t st_upb = size0 / 16;
        // (a round between planes only is dense on both sides as it is: the plain kernel, plane after plane)
        bool all_planes = pl.algorithm == ISO_ALG_COMBINED_STAGED && !deliver && uniform && !c.mesh;
        for (const HostEntry &he : ents)
            all_planes = all_planes && he.de.src_stride == size0 && he.de.dst_stride == size0;
        const bool staged_round = pl.algorithm == ISO_ALG_COMBINED_STAGED && !deliver && !all_planes && uniform &&
                                  size0 % 16 == 0 &&
                                  !lay.slot_major && !c.mesh && r.kind != ISO_ROUND_VECTOR && done == 0 &&
                                  ents.size() <= kLdsEntries && ents.size() * st_upb <= kTileUnits &&
                                  p * st_upb <= kMaxUnits;
        if (deliver) {
            deliver_launch(pd, ents, k, total);
        } else if (staged_round) {
            staged_round_launch(pd, r, ents, k, total);
        } else if (uniform && (!c.mesh || r.kind != ISO_ROUND_VECTOR)) {
            const int st = regular_launch(pd, r, ents, done, all_planes, k, total);
            if (st != ISO_SUCCESS) return st;
        } else {
            const int st = block_launch(pd, r, ents, done, k, total);
            if (st != ISO_SUCCESS) return st;
        }
        // streaming loads: all-to-all shift rounds of equal blocks (irregular blocks and the
        // s-exchange kernels are faster with cacheable loads)
        l.stream_loads = op == ISO_OP_ALLTOALL && r.kind != ISO_ROUND_VECTOR &&
                         (l.kernel == kShiftKernel || l.kernel == kMeshShiftKernel || l.kernel == kStagedRoundKernel ||
                          l.kernel == kDeliverKernel ||
                          (l.kernel == kBlockKernel && l.block.equal_units));
        std::vector<Side> src_sides, dst_sides;
        for (uint32_t q = 0; q < k; ++q) {
            const HostEntry &he = ents[done + q];
            src_sides.push_back(Side{he.de.src, he.de.src_stride, he.size});
            dst_sides.push_back(Side{he.de.dst, he.de.dst_stride, he.size});
        }
        set_grid(l, (uint32_t)total, k, page_resonant(src_sides) || page_resonant(dst_sides));
        pending.push_back(pd);
        done += k;
        return ISO_SUCCESS;
    }

    // Staged schedule, last launch: every rank's receive row written in one piece.
    void deliver_launch(Pending &pd, const std::vector<HostEntry> &ents, uint32_t &k, uint64_t &total) {
        Launch &l = pd.l;
        l.kernel = kDeliverKernel;
        DeliverArgs &da = l.deliver;
        const uint64_t upb = size0 / 16;
        k = (uint32_t)s;
        da.p = (uint32_t)p;
        da.s = (uint32_t)s;
        da.upb = (uint32_t)upb;
        l.tile_units = s * upb <= kSmallTileUnits ? kSmallTileUnits : kTileUnits;
        da.ranks = (uint32_t)std::min<uint64_t>(p, l.tile_units / (s * upb));
        da.dst = (uint64_t)(uintptr_t)recvbuf;
        while (prefixes.size() % 4) prefixes.push_back(0);            // 16-byte aligned entries
        pd.first_prefix = prefixes.size();
        for (int rows = 1; rows >= 0; --rows)                          // rank-major sources first
            for (const HostEntry &he : ents) {
                if ((he.de.src_stride > size0) != (rows == 1)) continue;
                const DeliverEntry x = make_deliver_entry(c, he);
                da.k_rows += rows == 1;
                const uint32_t *words = (const uint32_t *)&x;
                prefixes.insert(prefixes.end(), words, words + sizeof(x) / 4);
                table.push_back(he.de);      // keeps the launch's entry count in step with the others
            }
        da.d_upb = make_fastdiv(da.upb);
        da.d_rows = make_fastdiv(std::max(1u, da.k_rows * da.upb));
        da.d_plane = make_fastdiv(da.ranks * da.upb);
        da.d_row = make_fastdiv((uint32_t)(s * upb));
        l.dyn_lds = (uint32_t)(s * ((uint64_t)da.ranks * da.upb + 1) * 16);
        total = ((p + da.ranks - 1) / da.ranks) * kThreads;      // set_grid: one workgroup per tile
    }

    // Staged schedule, a round of small equal blocks: re-tiled through LDS.
    void staged_round_launch(Pending &pd, const Round &r, const std::vector<HostEntry> &ents, uint32_t &k,
                             uint64_t &total) {
        Launch &l = pd.l;
        l.kernel = kStagedRoundKernel;
        k = (uint32_t)ents.size();
        StagedRoundArgs &sa = l.staged;
        const uint64_t upb = size0 / 16;
        // entries that read a rank-major buffer (rank stride larger than the block) first
        for (int rows = 1; rows >= 0; --rows)
            for (const HostEntry &he : ents)
                if ((he.de.src_stride > size0) == (rows == 1)) {
                    table.push_back(he.de);
                    sa.k_rows += rows == 1;
                }
        sa.p = (uint32_t)p;
        sa.k = k;
        sa.upb = (uint32_t)upb;
        l.tile_units = k * upb <= kSmallTileUnits ? kSmallTileUnits : kTileUnits;
        sa.ranks = (uint32_t)std::min<uint64_t>(p, l.tile_units / (k * upb));
        const bool shift = r.kind == ISO_ROUND_SHIFT;
        sa.inner = shift ? (uint32_t)c.inner[r.dim] : 1u;
        sa.pj = shift ? (uint32_t)c.dims[r.dim] : 1u;
        sa.d_upb = make_fastdiv(sa.upb);
        sa.d_row = make_fastdiv(std::max(1u, sa.k_rows * sa.upb));
        sa.d_plane = make_fastdiv(sa.ranks * sa.upb);
        sa.d_inner = make_fastdiv(sa.inner);
        sa.d_pj = make_fastdiv(sa.pj);
        l.dyn_lds = (uint32_t)(k * ((uint64_t)sa.ranks * sa.upb + 1) * 16);
        total = ((p + sa.ranks - 1) / sa.ranks) * kThreads;      // set_grid: one workgroup per tile
    }

    // Regular blocks: every entry has `chunks` units of the request's common width (on a mesh: shift
    // rounds and same-rank copies; its s-exchange uses the block kernel).
    int regular_launch(Pending &pd, const Round &r, const std::vector<HostEntry> &ents, size_t done,
                       bool all_planes, uint32_t &k, uint64_t &total) {
        Launch &l = pd.l;
        const uint64_t width = uint64_t(1) << min_log2;
        const uint64_t chunks = (size0 + width - 1) >> min_log2;
        l.tail = (size0 & (width - 1)) != 0;
        const uint64_t per_entry = p * chunks;
        if (chunks > 0x7FFFFFFFu || per_entry > kMaxUnits) return ISO_ERR_TOO_LARGE;
        k = (uint32_t)std::min<uint64_t>(kMaxUnits / per_entry, ents.size() - done);
        total = per_entry * k;
        l.kernel = r.kind == ISO_ROUND_VECTOR ? kVectorKernel : c.mesh ? kMeshShiftKernel : kShiftKernel;
        // one block per wavefront: blocks that are a multiple of 1 KiB; on rank-major buffers only up
        // to 2 KiB (measured: no gain from 4 KiB on)
        l.uniform_waves = l.kernel == kShiftKernel && min_log2 == 4 && !l.tail && chunks % 64 == 0 &&
                          (lay.slot_major || chunks <= 128);
        const FastDiv dch = make_fastdiv((uint32_t)chunks), dk = make_fastdiv(k);
        const FastDiv dp = make_fastdiv((uint32_t)p);
        const bool shift = r.kind == ISO_ROUND_SHIFT;
        if (l.kernel == kVectorKernel) {
            l.vec.d = c.d;
            l.vec.d_chunks = dch;
            l.vec.d_k = dk;
            l.vec.d_p = dp;
            l.vec.entry_major = lay.slot_major || all_planes;
            l.vec.last_offset = size0 - width;
            for (int j = 0; j < c.d; ++j) {
                l.vec.d_dims[j] = make_fastdiv((uint32_t)c.dims[j]);
                l.vec.inner[j] = (uint32_t)c.inner[j];
            }
        } else if (l.kernel == kMeshShiftKernel) {
            MeshArgs &ma = l.mesh_shift;
            ma.inner = shift ? (uint32_t)c.inner[r.dim] : 1u;
            ma.pj = shift ? (uint32_t)c.dims[r.dim] : 1u;
            ma.shift_dim = shift ? r.dim : -1;
            ma.d = c.d;
            ma.d_chunks = dch;
            ma.d_k = dk;
            ma.d_p = dp;
            ma.entry_major = lay.slot_major;
            ma.last_offset = size0 - width;
            ma.d_inner = make_fastdiv(ma.inner);
            ma.d_pj = make_fastdiv(ma.pj);
            for (int j = 0; j < c.d; ++j) {
                if (c.periodic[(size_t)j]) ma.periodic_mask |= 1u << j;
                ma.d_dims[j] = make_fastdiv((uint32_t)c.dims[j]);
                ma.inner_of[j] = (uint32_t)c.inner[j];
            }
            const std::vector<uint32_t> bits =
                mesh_interior_tiles(c, lay.slot_major, ents.data() + done, k, total, chunks, p);
            prefixes.insert(prefixes.end(), bits.begin(), bits.end());
        } else {
            l.shift.inner = shift ? (uint32_t)c.inner[r.dim] : 1u;
            l.shift.pj = shift ? (uint32_t)c.dims[r.dim] : 1u;
            l.shift.d_chunks = dch;
            l.shift.d_k = dk;
            l.shift.d_p = dp;
            l.shift.entry_major = lay.slot_major || all_planes;
            // blocks of 2 KiB and more on rank-major buffers: groups of 64 ranks (three tori: 2 KiB -1 to
            // -3 % of the step, 4 KiB 0 to -3 %, 8 KiB -5 %; at 1 KiB and below between -1.5 and +1 %:
            // left alone.  Groups of 32 to 256 ranks measure alike, smaller ones do nothing)
            constexpr uint32_t kRankGroup = 64;
            if (!l.shift.entry_major && size0 >= 2048 && p >= kRankGroup) {
                l.shift.group = kRankGroup;
                l.shift.grouped = (uint32_t)((p / kRankGroup) * kRankGroup * k);
                l.shift.d_group_k = make_fastdiv(kRankGroup * k);
                l.shift.d_group = make_fastdiv(kRankGroup);
            }
            l.shift.last_offset = size0 - width;
            l.shift.d_inner = make_fastdiv(l.shift.inner);
            l.shift.d_pj = make_fastdiv(l.shift.pj);
        }
        for (uint32_t q = 0; q < k; ++q) table.push_back(ents[done + q].de);
        return ISO_SUCCESS;
    }

    // Irregular blocks, or a mesh's s-exchange: as many entries as fit the 32-bit unit index.
    int block_launch(Pending &pd, const Round &r, const std::vector<HostEntry> &ents, size_t done, uint32_t &k,
                     uint64_t &total) {
        Launch &l = pd.l;
        l.kernel = kBlockKernel;
        l.mesh = c.mesh;
        BlockArgs &b = l.block;
        b.shift_dim = r.kind == ISO_ROUND_SHIFT ? r.dim : -1;
        for (int j = 0; j < c.d; ++j)
            if (c.periodic[(size_t)j]) b.periodic_mask |= 1u << j;
        // per launch: k + 1 prefix values, then k multipliers of the divisions by the entries'
        // unit counts (the two shifts of each go into the entry's meta word)
        const bool entry_major = lay.slot_major;
        const uint64_t scale = entry_major ? p : 1;    // prefix counts all ranks' units, or one row's
        uint64_t row_units = 0;
        prefixes.push_back(0);
        while (done + k < ents.size()) {
            const uint64_t next = row_units + ents[done + k].de.units;
            if (next * p > kMaxUnits) break;
            row_units = next;
            DevEntry de = ents[done + k].de;
            const FastDiv by_units = make_fastdiv(de.units);
            de.meta |= (by_units.sh1 << 24) | (by_units.sh2 << 25);
            table.push_back(de);
            prefixes.push_back((uint32_t)(row_units * scale));
            ++k;
        }
        if (k == 0) return ISO_ERR_TOO_LARGE;          // one block plane alone is too large
        for (uint32_t q = 0; q < k; ++q) prefixes.push_back(make_fastdiv(ents[done + q].de.units).mul);
        total = row_units * p;
        b.entry_major = entry_major;
        b.equal_units = ents[done].de.units;
        for (uint32_t q = 1; q < k; ++q)
            if (ents[done + q].de.units != b.equal_units) b.equal_units = 0;
        b.d_units = make_fastdiv(b.equal_units ? b.equal_units : 1u);
        b.d_plane = make_fastdiv(b.equal_units ? (uint32_t)(p * b.equal_units) : 1u);
        b.vector_round = r.kind == ISO_ROUND_VECTOR;
        b.d_row = make_fastdiv((uint32_t)row_units);
        // shift rounds on rank-major buffers: ranks in groups (not the staged schedule, whose tiny
        // blocks travel through dense planes: +1 % there; not the s-exchange: +1 to +4 %)
        if (!entry_major && r.kind != ISO_ROUND_VECTOR && pl.algorithm != ISO_ALG_COMBINED_STAGED &&
            p >= kBlockGroup) {
            l.block_groups = true;
            b.grouped = (uint32_t)((p / kBlockGroup) * kBlockGroup * row_units);
            b.d_group_row = make_fastdiv((uint32_t)(row_units * kBlockGroup));
            b.d_plane = make_fastdiv(b.equal_units ? kBlockGroup * b.equal_units : 1u);
        }
        const bool shift = r.kind == ISO_ROUND_SHIFT;
        b.inner = shift ? (uint32_t)c.inner[r.dim] : 1u;
        b.pj = shift ? (uint32_t)c.dims[r.dim] : 1u;
        b.d_inner = make_fastdiv(b.inner);
        b.d_pj = make_fastdiv(b.pj);
        b.d = c.d;
        for (int j = 0; j < c.d; ++j) {
            b.d_dims[j] = make_fastdiv((uint32_t)c.dims[j]);
            b.inner_of[j] = (uint32_t)c.inner[j];
        }
        return ISO_SUCCESS;
    }

    // One device table: the entries, then the [s][d] residues, then what single launches read besides
    // (prefix arrays of irregular launches, the mesh's interior-tile bitmaps, the records of the staged
    // schedule's last launch); then the launches get their addresses in it.
    int upload() {
        const size_t entry_bytes = table.size() * sizeof(DevEntry);
        const size_t off_used = c.can.size() * sizeof(uint32_t);
        const size_t off_bytes = (off_used + 15) & ~size_t(15);     // what follows starts 16-byte aligned
        const size_t pre_bytes = prefixes.size() * sizeof(uint32_t);
        char *dev = nullptr;
        int st;
        if (arena) {
            if (entry_bytes + off_bytes + pre_bytes > arena->table_bytes) return ISO_ERR_SCRATCH;
            dev = (char *)arena->table;
            if ((st = store_table(*arena, 0, table.data(), entry_bytes)) != ISO_SUCCESS) return st;
            if ((st = store_table(*arena, entry_bytes, c.can.data(), off_used)) != ISO_SUCCESS) return st;
            if ((st = store_table(*arena, entry_bytes + off_bytes, prefixes.data(), pre_bytes)) != ISO_SUCCESS) return st;
        } else if (entry_bytes + off_bytes + pre_bytes) {
            ISO_HIP_TRY(hipMalloc(&rq.dev_table, entry_bytes + off_bytes + pre_bytes));
            dev = (char *)rq.dev_table;
            if (entry_bytes) ISO_HIP_TRY(hipMemcpy(dev, table.data(), entry_bytes, hipMemcpyHostToDevice));
            if (off_used) ISO_HIP_TRY(hipMemcpy(dev + entry_bytes, c.can.data(), off_used, hipMemcpyHostToDevice));
            if (pre_bytes)
                ISO_HIP_TRY(hipMemcpy(dev + entry_bytes + off_bytes, prefixes.data(), pre_bytes, hipMemcpyHostToDevice));
        }
        const DevEntry *dev_entries = (const DevEntry *)dev;
        const uint32_t *dev_offsets = (const uint32_t *)(dev + entry_bytes);
        const uint32_t *dev_prefix = (const uint32_t *)(dev + entry_bytes + off_bytes);
        for (Pending &pd : pending) {
            if (pd.l.kernel == kVectorKernel) {
                pd.l.vec.entries = dev_entries + pd.first_entry;
                pd.l.vec.offsets = dev_offsets;
            } else if (pd.l.kernel == kMeshShiftKernel) {
                pd.l.mesh_shift.entries = dev_entries + pd.first_entry;
                pd.l.mesh_shift.offsets = dev_offsets;
                pd.l.mesh_shift.interior = dev_prefix + pd.first_prefix;
            } else if (pd.l.kernel == kDeliverKernel) {
                pd.l.deliver.entries = (const DeliverEntry *)(dev_prefix + pd.first_prefix);
            } else if (pd.l.kernel == kStagedRoundKernel) {
                pd.l.staged.entries = dev_entries + pd.first_entry;
            } else if (pd.l.kernel == kBlockKernel) {
                pd.l.block.entries = dev_entries + pd.first_entry;
                pd.l.block.prefix = dev_prefix + pd.first_prefix;
                pd.l.block.offsets = dev_offsets;
            } else {
                pd.l.shift.entries = dev_entries + pd.first_entry;
            }
            rq.launches.push_back(pd.l);
        }
        inf.launches = (int32_t)rq.launches.size();
        return ISO_SUCCESS;
    }
};

inline int bind_request(BoundRequest &rq, const Comm &c, const Layout &lay, const void *sendbuf,
                        void *recvbuf, void *workspace, size_t workspace_bytes,
                        const StaticArena *arena = nullptr) {
    return Binder(rq, c, lay, sendbuf, recvbuf, workspace, workspace_bytes, arena).run();
}

}  // namespace iso
