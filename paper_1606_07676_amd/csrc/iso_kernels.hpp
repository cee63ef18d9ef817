// gfx950 kernels for isomorphic sparse collectives: pure data movement.
//
// One launch executes one round of a schedule: for every rank R and every entry
// e of the round it copies one block of m bytes
//
//     dst_e[R]  <-  src_e[ source rank of R ]
//
// where the source rank is R moved back v_e steps along one torus dimension
// (message-combining rounds, Section 5 / Algorithm 1 of the paper), R itself
// (zero offsets), or R (-) C^e (the straightforward exchange of Section 3).
// Entries carry absolute block addresses for rank 0 and the byte stride between
// consecutive ranks, so the same kernel reads and writes the user's rank-major
// [p][s][m] buffers and the workspace without pack or unpack copies.
//
// Work decomposition: the launch is a flat array of `vector-width` byte units
// ordered (rank, entry, chunk-in-block), chunk fastest, ONE unit per lane
// (slot-major buffers, one plane of p blocks per neighbour: (entry, rank, chunk),
// so that every wavefront access is one dense kilobyte of one plane).
// Consecutive lanes touch consecutive 16-byte pieces of one block, then the next
// block of the same rank: every wavefront load/store covers whole blocks, and a
// 256-lane workgroup covers 4 KiB of consecutive units.  Measured on MI355X,
// one unit per lane with the maximum number of resident wavefronts beats any
// per-lane unrolling (2, 4, 8 units per lane lose 3 %, 15 %, 50 %), for plain
// copies as well as for these gathers.  Stores are streaming (non-temporal):
// a block written in one round is next touched a whole round later (+8 % on
// the all-to-all rounds).  Loads are streaming too in the message-combining
// rounds of an all-to-all, where every source block is read exactly once
// (+1 to +9 %).  Everything else keeps cacheable loads: allgather rounds read
// one source block for several entries (streaming loads cost them 15 %), and
// the s-exchange kernels lose 25 % with streaming loads where the buffers fit
// the last-level cache and gain nothing where they do not.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "iso.h"
#include "iso_fastdiv.hpp"

namespace iso {

constexpr int kThreads = 256;
constexpr uint32_t kLdsEntries = 128;   // rounds with at most this many entries stage their table in LDS

struct alignas(16) DevEntry {
    uint64_t src;          // address of rank 0's source block
    uint64_t dst;          // address of rank 0's destination block
    uint32_t src_stride;   // bytes between consecutive ranks in the source buffer; below 2^32 (checked
    uint32_t dst_stride;   // when the request is bound), so that rank * stride + base is one 32x32+64 multiply-add
    uint32_t shift;        // SHIFT rounds: residue v; VECTOR rounds: neighbour index
    uint32_t units;        // block launches: units of this entry's block, block size / unit width rounded up
    uint32_t meta;         // block launches: bits 0-7 log2 of the unit width in bytes;
                           // bits 8-23 (mesh) dimensions in which R - C^ref must be inside the mesh;
                           // bits 24-29 the two shifts of the division by `units` (entry-major order)
    uint32_t ref;          // mesh: neighbour whose coordinates decide whether the move happens
    uint64_t last_offset;  // block launches: block size - unit width, the byte offset of the last unit
};

// Workgroup -> tile mapping.  The hardware hands consecutive workgroup ids to
// the 8 XCDs round-robin; each XCD has its own L2.  `run_log2` makes XCD x work
// on runs of 2^run_log2 consecutive tiles (tile = 256 consecutive units), the 8
// XCDs' runs interleaved, so that one L2 sees consecutive ranks while the 8 XCDs
// still sweep the same region of memory together.  kEighths instead gives XCD x
// the x-th contiguous eighth of all tiles: the host picks it for launches whose
// blocks sit at rank strides that are multiples of 4 KiB and cover only part of a
// 4 KiB page (see page_resonant), where it is 4 - 26 % faster.
struct TileMap {
    uint32_t n_tiles;      // tiles that carry work
    uint32_t run_log2;     // kEighths: XCD x works on the x-th contiguous eighth of the tiles
    uint32_t per_xcd;      // kEighths: tiles per XCD, ceil(n_tiles / 8)
};
constexpr uint32_t kEighths = 31;

__device__ __forceinline__ bool tile_of_block(const TileMap &tm, uint32_t &tile) {
    const uint32_t bid = blockIdx.x, x = bid & 7u, y = bid >> 3;
    if (tm.run_log2 == kEighths) tile = x * tm.per_xcd + y;
    else tile = ((y >> tm.run_log2) << (tm.run_log2 + 3)) + (x << tm.run_log2) + (y & ((1u << tm.run_log2) - 1u));
    return tile < tm.n_tiles;
}

struct ShiftArgs {
    const DevEntry *entries;
    TileMap map;
    uint32_t total;        // units in this launch = p * k * chunks
    uint32_t k;            // entries in this launch
    uint32_t inner;        // rank stride of the shifted dimension
    uint32_t pj;           // its size
    uint32_t entry_major;  // unit order (entry, rank, chunk) instead of (rank, entry, chunk)
    FastDiv d_chunks, d_k, d_inner, d_pj, d_p;
    uint64_t last_offset;  // block size - unit width (read by the TAIL instantiations only)
    // Large blocks on rank-major buffers: the ranks are taken in groups of `group`, and inside a group the
    // order is (entry, rank, chunk), so that a plane of the workspace sees `group` consecutive blocks at a
    // time instead of one (0: no groups).  `grouped` = the blocks of all whole groups, (p / group) * group * k;
    // the ranks after them keep the plain order.
    uint32_t group, grouped;
    FastDiv d_group_k, d_group;   // group * k; group
};

struct VectorArgs {
    const DevEntry *entries;
    const uint32_t *offsets;   // [s][d] residues
    TileMap map;
    uint32_t total;
    uint32_t k;
    int32_t d;
    uint32_t entry_major;
    FastDiv d_chunks, d_k, d_p;
    FastDiv d_dims[ISO_MAX_DIMS];
    uint32_t inner[ISO_MAX_DIMS];
    uint64_t last_offset;
};

typedef uint32_t vec16_t __attribute__((ext_vector_type(4)));
typedef uint32_t vec8_t __attribute__((ext_vector_type(2)));

// A block of `size` bytes is moved in units of w bytes, w the largest power of two that is at
// most 16 and at most `size`: ceil(size / w) units, unit c at byte offset min(c * w, size - w).
// When w does not divide the size the last unit overlaps the one before it; both carry the same
// bytes of the same block, so the doubly written bytes get the same value twice.  Addresses
// need no alignment: the unit types are declared with alignment 1 and global memory accesses of
// any width take any address on this target.
template <typename V>
struct Unaligned {
    typedef V type __attribute__((aligned(1)));
};

// The unit at byte offset `off` of the block at byte address `src` to the same offset of the
// block at `dst`, both in global memory (the address space is spelled out so that the accesses
// are global_load / global_store, not flat ones).  NTL: streaming load.
template <typename V, bool NTL>
__device__ __forceinline__ void move_unit(uint64_t dst, uint64_t src, uint64_t off) {
    typedef typename Unaligned<V>::type UV;
    typedef const UV __attribute__((address_space(1))) *src_ptr;
    typedef UV __attribute__((address_space(1))) *dst_ptr;
    const src_ptr sp = (src_ptr)(src + off);
    V v;
    if constexpr (NTL) v = __builtin_nontemporal_load(sp);
    else v = *sp;
    // Streaming stores for 16-byte units only.  Narrower units belong to blocks of a few bytes, of
    // which several wavefronts write different bytes of one cache line: plain stores let the L2
    // merge them before the line goes to memory.
    if constexpr (sizeof(V) == 16) __builtin_nontemporal_store(v, (dst_ptr)(dst + off));
    else *(dst_ptr)(dst + off) = v;
}

template <typename V>
__device__ __forceinline__ uint64_t unit_offset(uint32_t ch, uint64_t last_offset) {
    const uint64_t off = (uint64_t)ch * sizeof(V);
    return off < last_offset ? off : last_offset;
}

// TAIL: the width does not divide the block size.  The regular kernels are instantiated
// without it as well: the comparison and selects cost 2 % on the round kernel.
template <typename V, bool TAIL>
__device__ __forceinline__ uint64_t unit_offset_if(uint32_t ch, uint64_t last_offset) {
    if constexpr (TAIL) return unit_offset<V>(ch, last_offset);
    else return (uint64_t)ch * sizeof(V);
}

// Address of rank R's block: base + R * stride with the stride known to fit 32 bits.
__device__ __forceinline__ uint64_t block_address(uint64_t base, uint32_t R, uint32_t stride) {
    return base + (uint64_t)R * stride;
}

// Entry table of the launch: from LDS (staged once per workgroup) when it fits,
// else straight from global memory (cached).
template <bool LDS>
struct EntryTable {
    const DevEntry *tab;
    __device__ __forceinline__ EntryTable(const DevEntry *global, uint32_t k, DevEntry *lds) {
        if constexpr (LDS) {
            if (threadIdx.x < k) lds[threadIdx.x] = global[threadIdx.x];
            __syncthreads();
            tab = lds;
        } else {
            tab = global;
        }
    }
    __device__ __forceinline__ DevEntry operator[](uint32_t e) const { return tab[e]; }
};

// The same staging in two steps, so that a kernel can put work that does not depend on the table
// between the table's load and its arrival in LDS: issue() starts the load of this lane's entry,
// commit() writes it to LDS and synchronises the workgroup.  (Three plain 16-byte registers: a
// DevEntry variable here ends up in LDS itself.)
template <bool LDS>
struct StagedEntries {
    static_assert(sizeof(DevEntry) == 48, "staged as three 16-byte words");
    vec16_t w0, w1, w2;
    bool mine;
    __device__ __forceinline__ void issue(const DevEntry *global, uint32_t k) {
        w0 = w1 = w2 = vec16_t{};
        mine = LDS && threadIdx.x < k;
        if (mine) {
            const vec16_t *from = (const vec16_t *)(global + threadIdx.x);
            w0 = from[0];
            w1 = from[1];
            w2 = from[2];
        }
    }
    __device__ __forceinline__ void commit(DevEntry *lds) const {
        if constexpr (LDS) {
            if (mine) {
                vec16_t *to = (vec16_t *)(lds + threadIdx.x);
                to[0] = w0;
                to[1] = w1;
                to[2] = w2;
            }
            __syncthreads();
        }
    }
};

// Coordinate decodes over all dimensions.  For d <= kUnrolledDims the code is instantiated
// for the exact d (one uniform switch, then straight-line code): the per-dimension launch
// constants are then read at fixed kernel-argument offsets (scalar registers) and the loads
// of the offset vector are issued together.  Indexing those arrays with a run-time j costs a
// dependent scalar load and several uniform branches per dimension, and at one unit per lane
// that is a third of the kernel's throughput.
// Rank arithmetic is done modulo 2^32: ranks are below 2^31 and every true result lies in
// [0, p), so wrapped intermediate values are harmless.
constexpr int kUnrolledDims = 6;

// Source rank of R for a move by the full offset vector c[0..d): R (-) c on the torus.
template <int D>
__device__ __forceinline__ uint32_t vector_source_rank_d(uint32_t R, const uint32_t *__restrict__ c,
                                                         const FastDiv (&d_dims)[ISO_MAX_DIMS],
                                                         const uint32_t (&inner)[ISO_MAX_DIMS]) {
    uint32_t cj[D];
#pragma unroll
    for (int j = 0; j < D; ++j) cj[j] = c[j];
    uint32_t srcR = R, rem = R;
#pragma unroll
    for (int j = D - 1; j >= 0; --j) {
        uint32_t q, rj;
        fast_divmod(rem, d_dims[j], q, rj);
        rem = q;
        srcR -= cj[j] * inner[j];                                   // cj steps back ...
        if (rj < cj[j]) srcR += d_dims[j].div * inner[j];           // ... around the ring
    }
    return srcR;
}

__device__ __forceinline__ uint32_t vector_source_rank(uint32_t R, const uint32_t *__restrict__ c, int32_t d,
                                                       const FastDiv (&d_dims)[ISO_MAX_DIMS],
                                                       const uint32_t (&inner)[ISO_MAX_DIMS]) {
    switch (d) {
        case 1: return vector_source_rank_d<1>(R, c, d_dims, inner);
        case 2: return vector_source_rank_d<2>(R, c, d_dims, inner);
        case 3: return vector_source_rank_d<3>(R, c, d_dims, inner);
        case 4: return vector_source_rank_d<4>(R, c, d_dims, inner);
        case 5: return vector_source_rank_d<5>(R, c, d_dims, inner);
        case 6: return vector_source_rank_d<6>(R, c, d_dims, inner);
        default: break;
    }
    uint32_t srcR = R, rem = R;
    for (int j = d - 1; j >= 0; --j) {
        uint32_t q, rj;
        fast_divmod(rem, d_dims[j], q, rj);
        rem = q;
        srcR -= c[j] * inner[j];
        if (rj < c[j]) srcR += d_dims[j].div * inner[j];
    }
    return srcR;
}

// Makes the compiler fetch these launch constants here, in one batch of scalar loads, instead of
// each in front of its first use behind some branch (every such fetch is a wait of its own).
__device__ __forceinline__ void fetch_now(const FastDiv &f) { asm volatile("" ::"s"(f.mul), "s"(f.sh1), "s"(f.sh2), "s"(f.div)); }

__device__ __forceinline__ void fetch_now(const ShiftArgs &a) {
    asm volatile("" ::"s"(a.entries), "s"(a.map.n_tiles), "s"(a.map.run_log2), "s"(a.map.per_xcd), "s"(a.total),
                 "s"(a.k), "s"(a.inner), "s"(a.pj), "s"(a.entry_major));
    fetch_now(a.d_chunks);
    fetch_now(a.d_k);
    fetch_now(a.d_inner);
    fetch_now(a.d_pj);
    fetch_now(a.d_p);
}

template <typename V, bool LDS, bool NTL, bool TAIL, bool GROUPS = false>
__global__ __launch_bounds__(kThreads) void shift_round_kernel(const ShiftArgs a) {
    fetch_now(a);
    if constexpr (GROUPS) {
        asm volatile("" ::"s"(a.group), "s"(a.grouped));
        fetch_now(a.d_group_k);
        fetch_now(a.d_group);
    }
    __shared__ DevEntry lds[LDS ? kLdsEntries : 1];
    uint32_t tile;
    if (!tile_of_block(a.map, tile)) return;            // (the whole workgroup: no one is left at the barrier)
    // The table goes through LDS; its load is under way while the lanes work out their indices, which do
    // not depend on it.
    StagedEntries<LDS> staging;
    staging.issue(a.entries, a.k);
    const uint32_t u = tile * (uint32_t)kThreads + threadIdx.x;
    uint32_t t, ch, R, e;
    fast_divmod(u, a.d_chunks, t, ch);
    if constexpr (GROUPS) {                             // an instantiation of its own: the few scalar loads and
        if (t < a.grouped) {                            // the branch cost the plain one 2 - 3 % on small blocks
            uint32_t g, in_group, rg;
            fast_divmod(t, a.d_group_k, g, in_group);
            fast_divmod(in_group, a.d_group, e, rg);
            R = g * a.group + rg;
        } else {
            fast_divmod(t - a.grouped, a.d_k, R, e);
            R += fast_div(a.grouped, a.d_k);            // the ranks of the whole groups come first
        }
    } else if (a.entry_major) {
        fast_divmod(t, a.d_p, e, R);
    } else {
        fast_divmod(t, a.d_k, R, e);
    }
    const uint32_t q = fast_div(R, a.d_inner);
    const uint32_t rj = q - fast_div(q, a.d_pj) * a.pj;       // coordinate of R in the shifted dimension
    staging.commit(lds);
    if (u >= a.total) return;                                  // (indices beyond the launch are never used)
    const DevEntry en = LDS ? lds[e] : a.entries[e];
    // v steps back along the dimension, around the ring where that passes coordinate 0 (modulo 2^32;
    // the true result lies in [0, p))
    uint32_t srcR = R - en.shift * a.inner;
    if (rj < en.shift) srcR += a.pj * a.inner;
    move_unit<V, NTL>(block_address(en.dst, R, en.dst_stride), block_address(en.src, srcR, en.src_stride),
                      unit_offset_if<V, TAIL>(ch, a.last_offset));
}

// The same round for blocks that are a multiple of 1 KiB (64 units of 16 bytes): the 64 units of a
// wavefront then belong to one block, so rank, entry and source rank are the same for all its lanes
// and are computed once, in scalar registers, the entry fetched with scalar loads.  No staging of the
// table through LDS, no barrier, no vector-memory access in front of the one load that matters: what
// bounds these kernels is how long a wavefront holds its slot before that load is under way.
template <bool NTL, bool GROUPS = false>
__global__ __launch_bounds__(kThreads) void shift_round_uniform_kernel(const ShiftArgs a) {
    fetch_now(a);
    uint32_t tile;
    if (!tile_of_block(a.map, tile)) return;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t u0 = tile * (uint32_t)kThreads + wave * 64u;      // first unit of this wavefront
    if (u0 >= a.total) return;                                       // total is a multiple of 64
    uint32_t t, ch0, R, e;
    fast_divmod(u0, a.d_chunks, t, ch0);
    if constexpr (GROUPS) {
        if (t < a.grouped) {
            uint32_t g, in_group, rg;
            fast_divmod(t, a.d_group_k, g, in_group);
            fast_divmod(in_group, a.d_group, e, rg);
            R = g * a.group + rg;
        } else {
            fast_divmod(t - a.grouped, a.d_k, R, e);
            R += fast_div(a.grouped, a.d_k);
        }
    } else if (a.entry_major) {
        fast_divmod(t, a.d_p, e, R);
    } else {
        fast_divmod(t, a.d_k, R, e);
    }
    const uint32_t q = fast_div(R, a.d_inner);
    const uint32_t rj = q - fast_div(q, a.d_pj) * a.pj;
    // the table is never written while a collective runs: read it as constant memory, through the scalar cache
    typedef const DevEntry __attribute__((address_space(4))) *const_entry_ptr;
    const const_entry_ptr en = (const_entry_ptr)(uintptr_t)(a.entries + e);
    const uint32_t shift = en->shift;
    uint32_t srcR = R - shift * a.inner;
    if (rj < shift) srcR += a.pj * a.inner;
    const uint64_t src = block_address(en->src, srcR, en->src_stride);
    const uint64_t dst = block_address(en->dst, R, en->dst_stride);
    move_unit<vec16_t, NTL>(dst, src, (uint64_t)(ch0 + (threadIdx.x & 63u)) * sizeof(vec16_t));
}

// (the decode constants of the first three dimensions with the rest: few tori have more, and each
// further dimension's are fetched where the decode reaches it)
__device__ __forceinline__ void fetch_now(const VectorArgs &a) {
    asm volatile("" ::"s"(a.entries), "s"(a.offsets), "s"(a.map.n_tiles), "s"(a.map.run_log2), "s"(a.map.per_xcd),
                 "s"(a.total), "s"(a.k), "s"(a.d), "s"(a.entry_major), "s"(a.inner[0]), "s"(a.inner[1]),
                 "s"(a.inner[2]));
    fetch_now(a.d_chunks);
    fetch_now(a.d_k);
    fetch_now(a.d_p);
    fetch_now(a.d_dims[0]);
    fetch_now(a.d_dims[1]);
    fetch_now(a.d_dims[2]);
}

template <typename V, bool LDS, bool TAIL>
__global__ __launch_bounds__(kThreads) void vector_round_kernel(const VectorArgs a) {
    fetch_now(a);
    __shared__ DevEntry lds[LDS ? kLdsEntries : 1];
    uint32_t tile;
    if (!tile_of_block(a.map, tile)) return;
    StagedEntries<LDS> staging;
    staging.issue(a.entries, a.k);
    const uint32_t u = tile * (uint32_t)kThreads + threadIdx.x;
    uint32_t t, ch, R, e;
    fast_divmod(u, a.d_chunks, t, ch);
    if (a.entry_major) fast_divmod(t, a.d_p, e, R);
    else fast_divmod(t, a.d_k, R, e);
    staging.commit(lds);
    if (u >= a.total) return;
    const DevEntry en = LDS ? lds[e] : a.entries[e];
    const uint32_t srcR = vector_source_rank(R, a.offsets + (size_t)en.shift * a.d, a.d, a.d_dims, a.inner);
    move_unit<V, false>(block_address(en.dst, R, en.dst_stride), block_address(en.src, srcR, en.src_stride),
                        unit_offset_if<V, TAIL>(ch, a.last_offset));
}

// Irregular blocks (the v/w interfaces of Section 2): every entry has its own
// block size and its own unit width (16 bytes for blocks of at least 16 bytes,
// narrower below, e.g. a 1-byte corner block next to a 16 KiB face block).
// A rank's units are the concatenation of its entries' units; `prefix[e]` is
// the first unit of entry e.  The flat index is split into (rank, unit in row),
// the entry is found by binary search in the prefix array.  On slot-major
// buffers (one plane of p blocks per neighbour) the order is (entry, rank, unit)
// instead: prefix[e] then counts the units of all ranks in the entries before e,
// and the position inside the plane is divided by the entry's own unit count.
// (Measured against this form and dropped: the launch cut into one segment per unit
// width, each a whole number of tiles, so that the width switch is uniform in a
// workgroup.  Selecting the segment's constants puts one more stage of dependent
// scalar loads in front of every wavefront's load: stencil-shaped all-to-all,
// 4096 / 64 / 1 byte blocks, -2 % on rank-major buffers, -15 % on slot-major ones,
// -11 % for the fused s-exchange.  What tiny blocks cost is not in the kernel: a
// block of a few bytes in every rank's row is a memory access of its own on each
// side, whatever moves it.)
//
// MESH (Section 7, non-periodic dimensions): coordinates of non-periodic
// dimensions are signed and nothing wraps there.  A move happens at rank R only
// if R - C^ref stays inside the mesh in every dimension of the entry's mask
// (the non-periodic dimensions routed up to and including this round in which
// C^ref is non-zero); otherwise the destination keeps its content.
struct BlockArgs {
    const DevEntry *entries;
    const uint32_t *prefix;    // [k + 1] first unit of every entry, then [k] multipliers (entry-major order)
    const uint32_t *offsets;   // [s][d] effective coordinates (residues; signed where non-periodic)
    TileMap map;
    uint32_t total;            // p * row_units
    uint32_t k;
    uint32_t vector_round;     // 0: shift along one dimension, 1: full offset vector
    uint32_t inner, pj;        // shift rounds
    int32_t shift_dim;         // shift rounds: the dimension (-1: same-rank copy)
    uint32_t periodic_mask;    // bit j set: dimension j wraps
    int32_t d;
    uint32_t equal_units;      // != 0: every entry of the launch has this many units (no search)
    uint32_t entry_major;      // slot-major buffers: units ordered (entry, rank, unit) and prefix[e] counts
                               // the units of all ranks before entry e; else (rank, entry, unit)
    uint32_t grouped;          // GROUPS: units of the ranks that form whole groups (the first ones)
    FastDiv d_row, d_inner, d_pj, d_units, d_plane;   // d_plane: p * equal_units (GROUPS: group * equal_units)
    FastDiv d_group_row;       // GROUPS: units of a group's rows
    FastDiv d_dims[ISO_MAX_DIMS];
    uint32_t inner_of[ISO_MAX_DIMS];
};

// Mesh: does the move of entry `en` happen at rank R (R - C^ref inside the mesh in every masked
// dimension), and from which rank?  Offsets of non-periodic dimensions are signed values stored
// as two's complement, so one unsigned comparison tests both ends of the dimension.
template <int D, typename Args>
__device__ __forceinline__ bool mesh_source_rank_d(const Args &a, const DevEntry &en, uint32_t R,
                                                   uint32_t &srcR) {
    const uint32_t mask = (en.meta >> 8) & 0xFFFFu;
    const uint32_t *cref = a.offsets + (size_t)en.ref * a.d;
    uint32_t cr[D], r[D];
#pragma unroll
    for (int j = 0; j < D; ++j) cr[j] = cref[j];
    uint32_t rem = R;
#pragma unroll
    for (int j = D - 1; j >= 0; --j) {
        uint32_t q;
        fast_divmod(rem, a.d_dims[j], q, r[j]);
        rem = q;
    }
    uint32_t outside = 0;
#pragma unroll
    for (int j = 0; j < D; ++j)
        outside |= ((mask >> j) & 1u) & (uint32_t)((uint32_t)(r[j] - cr[j]) >= a.d_dims[j].div);
    if (outside) return false;
    srcR = R;
    if (a.vector_round) {                                  // en.shift: the neighbour whose offsets move the block
        const uint32_t *cvec = a.offsets + (size_t)en.shift * a.d;
        uint32_t cv[D];
#pragma unroll
        for (int j = 0; j < D; ++j) cv[j] = cvec[j];
#pragma unroll
        for (int j = 0; j < D; ++j) {
            srcR -= cv[j] * a.inner_of[j];                 // signed where the dimension does not wrap
            if (((a.periodic_mask >> j) & 1u) && r[j] < cv[j]) srcR += a.d_dims[j].div * a.inner_of[j];
        }
    } else if (a.shift_dim >= 0) {                         // en.shift: the distance along the one moving dimension
        uint32_t rj = 0;
#pragma unroll
        for (int j = 0; j < D; ++j)
            if (j == a.shift_dim) rj = r[j];                // uniform condition: a select, not a branch per lane
        srcR -= en.shift * a.inner;
        if (((a.periodic_mask >> a.shift_dim) & 1u) && rj < en.shift) srcR += a.pj * a.inner;
    }
    return true;
}

template <typename Args>
__device__ __forceinline__ bool mesh_source_rank(const Args &a, const DevEntry &en, uint32_t R,
                                                 uint32_t &srcR) {
    switch (a.d) {
        case 1: return mesh_source_rank_d<1>(a, en, R, srcR);
        case 2: return mesh_source_rank_d<2>(a, en, R, srcR);
        case 3: return mesh_source_rank_d<3>(a, en, R, srcR);
        case 4: return mesh_source_rank_d<4>(a, en, R, srcR);
        case 5: return mesh_source_rank_d<5>(a, en, R, srcR);
        case 6: return mesh_source_rank_d<6>(a, en, R, srcR);
        default: break;
    }
    // more dimensions: one pass with run-time indices
    const uint32_t mask = (en.meta >> 8) & 0xFFFFu;
    const uint32_t *cref = a.offsets + (size_t)en.ref * a.d;
    // in shift rounds en.shift is the distance itself: no row of the offset table is addressed with it
    const uint32_t *cvec = a.vector_round ? a.offsets + (size_t)en.shift * a.d : cref;
    uint32_t rem = R;
    bool has_source = true;
    srcR = R;
    for (int j = a.d - 1; j >= 0; --j) {
        uint32_t q, rj;
        fast_divmod(rem, a.d_dims[j], q, rj);
        rem = q;
        const uint32_t pj = a.d_dims[j].div;
        if (((mask >> j) & 1u) && (uint32_t)(rj - cref[j]) >= pj) has_source = false;
        if (a.vector_round || j == a.shift_dim) {
            const uint32_t cj = a.vector_round ? cvec[j] : en.shift;
            srcR -= cj * a.inner_of[j];
            if (((a.periodic_mask >> j) & 1u) && rj < cj) srcR += pj * a.inner_of[j];
        }
    }
    return has_source;
}

// GROUPS (rank-major buffers, shift rounds): the ranks are taken in groups of kBlockGroup, and inside
// a group the units are ordered (entry, rank, unit) as on slot-major buffers, so that large and tiny
// blocks fall into different workgroups and a workgroup's wide units are not held up by a second
// pass for narrow ones; prefix[] still counts one row's units.  Ranks beyond the last whole group
// are taken one by one.  (Stencil-shaped all-to-all on 32 x 32 x 32, blocks of 4096 / 64 / 1 bytes:
// groups of 8 ranks -4 % of the step, 32 -5 %, 64 -6.5 %, 128 and 256 -7.5 %, 1024 -7 %.)
constexpr uint32_t kBlockGroupLog2 = 7, kBlockGroup = 1u << kBlockGroupLog2;

__device__ __forceinline__ void fetch_now(const BlockArgs &a) {
    asm volatile("" ::"s"(a.entries), "s"(a.prefix), "s"(a.map.n_tiles), "s"(a.map.run_log2), "s"(a.map.per_xcd),
                 "s"(a.total), "s"(a.k), "s"(a.vector_round), "s"(a.inner), "s"(a.pj), "s"(a.equal_units),
                 "s"(a.entry_major), "s"(a.grouped));
    fetch_now(a.d_row);
    fetch_now(a.d_inner);
    fetch_now(a.d_pj);
    fetch_now(a.d_units);
    fetch_now(a.d_plane);
    fetch_now(a.d_group_row);
}

template <bool LDS, bool MESH, bool NTL, bool GROUPS = false>
__global__ __launch_bounds__(kThreads) void block_round_kernel(const BlockArgs a) {
    if constexpr (!MESH) fetch_now(a);
    __shared__ DevEntry lds[LDS ? kLdsEntries : 1];
    __shared__ uint32_t lds_prefix[LDS ? 2 * kLdsEntries + 1 : 1];
    const uint32_t *prefix = a.prefix;
    if constexpr (LDS) {
        // staged by the workgroup's last lanes, the entries (below) by its first: with few entries these are
        // different wavefronts, and the two loads are in flight together
        for (uint32_t q = kThreads - 1 - threadIdx.x; q <= 2 * a.k; q += kThreads) lds_prefix[q] = a.prefix[q];
        prefix = lds_prefix;
    }
    const EntryTable<LDS> table(a.entries, a.k, lds);     // synchronises the workgroup when LDS
    // (the two-step staging of the other kernels, with the first division between the steps, is 0.5 to 1 %
    // slower here)
    uint32_t tile;
    if (!tile_of_block(a.map, tile)) return;
    const uint32_t u = tile * (uint32_t)kThreads + threadIdx.x;
    if (u >= a.total) return;
    // flat index -> rank R, entry lo, unit ch of that entry's block
    uint32_t R = 0, lo = 0, ch = 0, w = u;
    uint32_t span_log2 = 0;                                // GROUPS: w counts through 2^span_log2 rows, entry by entry
    bool planes = a.entry_major;                           // w (then ch) counts through several ranks' blocks
    if constexpr (GROUPS) {
        planes = u < a.grouped;
        if (planes) {
            fast_divmod(u, a.d_group_row, R, w);          // R: the group, below its first rank
            R <<= kBlockGroupLog2;
            span_log2 = kBlockGroupLog2;
        } else {
            fast_divmod(u - a.grouped, a.d_row, R, w);
            R += fast_div(a.grouped, a.d_row);
        }
    } else if (!a.entry_major) {
        fast_divmod(u, a.d_row, R, w);                     // w: unit inside the rank's row
    }
    // entry-major: w counts through the entries one after another, each with the units of all p ranks
    if (a.k == 1) {
        ch = w;
    } else if (a.equal_units) {                            // equal blocks: plain division, no search
        fast_divmod(w, planes ? a.d_plane : a.d_units, lo, ch);
    } else {
        const uint32_t key = w >> span_log2;               // prefix[e] * 2^n <= w  <=>  prefix[e] <= w >> n
        uint32_t hi = a.k;                                 // largest e with prefix[e] <= key
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (prefix[mid] <= key) lo = mid;
            else hi = mid;
        }
        ch = w - (prefix[lo] << span_log2);
    }
    const DevEntry en = table[lo];
    if (planes) {                                          // ch still counts (rank, unit) inside the plane
        const FastDiv by_units = a.equal_units
                                     ? a.d_units
                                     : FastDiv{prefix[a.k + 1 + lo], (en.meta >> 24) & 1u, (en.meta >> 25) & 31u, en.units};
        const uint32_t in_plane = ch;
        uint32_t rank_in_span;
        fast_divmod(in_plane, by_units, rank_in_span, ch);
        R += rank_in_span;
    }
    uint32_t srcR = R;                                    // modulo 2^32, see vector_source_rank
    if constexpr (MESH) {
        if (!mesh_source_rank(a, en, R, srcR)) return;    // no source: leave the destination as it is
    } else if (a.vector_round) {
        srcR = vector_source_rank(R, a.offsets + (size_t)en.shift * a.d, a.d, a.d_dims, a.inner_of);
    } else {
        const uint32_t q = fast_div(R, a.d_inner);
        const uint32_t rj = q - fast_div(q, a.d_pj) * a.pj;
        srcR -= en.shift * a.inner;
        if (rj < en.shift) srcR += a.pj * a.inner;
    }
    const uint64_t src = block_address(en.src, srcR, en.src_stride);
    const uint64_t dst = block_address(en.dst, R, en.dst_stride);
    switch (en.meta & 0xFFu) {
        case 4: move_unit<vec16_t, NTL>(dst, src, unit_offset<vec16_t>(ch, en.last_offset)); break;
        case 3: move_unit<vec8_t, false>(dst, src, unit_offset<vec8_t>(ch, en.last_offset)); break;
        case 2: move_unit<uint32_t, false>(dst, src, unit_offset<uint32_t>(ch, en.last_offset)); break;
        case 1: move_unit<uint16_t, false>(dst, src, unit_offset<uint16_t>(ch, en.last_offset)); break;
        default: move_unit<uint8_t, false>(dst, src, ch); break;
    }
}

// Shift rounds of equal blocks on a mesh: the shift kernel's decomposition (no prefix search, no
// per-entry unit width) with the mesh's validity test.  Field names match what mesh_source_rank reads.
//
// Most ranks of a mesh are interior: every move of the launch has a source there.  The host marks,
// one bit per tile, the tiles all of whose ranks are interior; such a workgroup skips the per-lane
// decode of all coordinates and the loads of the reference offsets and does what the torus kernel
// does.  (Deciding this in the kernel from the tile's first and last rank costs as much as it
// saves: the test is a chain of dependent scalar loads of launch constants, and what bounds these
// kernels is how long a wavefront holds its slot before its one load is under way.)
struct MeshArgs {
    const DevEntry *entries;
    const uint32_t *offsets;   // [s][d] effective coordinates
    const uint32_t *interior;  // bit t: every rank of tile t has a source for every entry of the launch
    TileMap map;
    uint32_t total, k;
    uint32_t inner, pj;        // rank stride and size of the moving dimension (1, 1 for a same-rank copy)
    uint32_t entry_major;
    int32_t shift_dim;         // -1: same-rank copy
    int32_t d;
    uint32_t periodic_mask;
    static constexpr uint32_t vector_round = 0;
    FastDiv d_chunks, d_k, d_p, d_inner, d_pj;
    FastDiv d_dims[ISO_MAX_DIMS];
    uint32_t inner_of[ISO_MAX_DIMS];
    uint64_t last_offset;
};

template <typename V, bool LDS, bool NTL, bool TAIL>
__global__ __launch_bounds__(kThreads) void mesh_shift_round_kernel(const MeshArgs a) {
    __shared__ DevEntry lds[LDS ? kLdsEntries : 1];
    uint32_t tile;
    if (!tile_of_block(a.map, tile)) return;
    StagedEntries<LDS> staging;
    staging.issue(a.entries, a.k);
    const bool interior = (a.interior[tile >> 5] >> (tile & 31u)) & 1u;      // uniform: one scalar load
    const uint32_t u = tile * (uint32_t)kThreads + threadIdx.x;
    uint32_t t, ch, R, e;
    fast_divmod(u, a.d_chunks, t, ch);
    if (a.entry_major) fast_divmod(t, a.d_p, e, R);
    else fast_divmod(t, a.d_k, R, e);
    staging.commit(lds);
    if (u >= a.total) return;
    const DevEntry en = LDS ? lds[e] : a.entries[e];
    uint32_t srcR = R;
    if (interior) {                                       // every move has its source: the torus kernel's path
        if (a.shift_dim >= 0) {
            srcR -= en.shift * a.inner;
            if ((a.periodic_mask >> a.shift_dim) & 1u) {  // the moving dimension wraps
                const uint32_t q = fast_div(R, a.d_inner);
                const uint32_t rj = q - fast_div(q, a.d_pj) * a.pj;
                if (rj < en.shift) srcR += a.pj * a.inner;
            }
        }
    } else if (!mesh_source_rank(a, en, R, srcR)) {
        return;                                           // no source: leave the destination as it is
    }
    move_unit<V, NTL>(block_address(en.dst, R, en.dst_stride), block_address(en.src, srcR, en.src_stride),
                      unit_offset_if<V, TAIL>(ch, a.last_offset));
}

// ---- small blocks re-tiled through LDS (the staged schedule) ----------------------------------
// A workgroup moves a tile of up to kTileUnits units: the blocks of `ranks` consecutive ranks for
// all entries of the launch.  It reads them in the order that suits the source (entry after entry
// of one rank where the source is a rank-major buffer, rank after rank of one plane where it is a
// slot-major one), eight independent loads per lane, parks them in LDS, and writes them in the
// order that suits the destination.  Both sides then see runs of hundreds of bytes although the
// blocks themselves may be 16 bytes.  In a round the tile's ranks are SOURCE ranks (the kernel
// pushes: block e of rank S goes to rank S + v_e), so that all pieces of one send-buffer row, those
// moving up and those moving down the dimension, are read by one workgroup and share their memory
// lines; every destination block is still written exactly once.  The last launch below tiles by
// destination rank instead, because it is the receive rows that it writes whole.
constexpr uint32_t kTileUnits = 2048;                  // the largest tile: 8 units per lane
constexpr uint32_t kSmallTileUnits = 1024;             // used where the blocks of one rank fit it: 3 % faster at 16-byte
                                                       // blocks, 2 % at 128 bytes (512: 4 % slower than 1024)

struct StagedRoundArgs {
    const DevEntry *entries;   // the first k_rows entries read a rank-major buffer, the others a slot-major one;
                               // every destination is a slot-major plane of the workspace
    TileMap map;
    uint32_t p, k, k_rows;
    uint32_t ranks;            // ranks per tile: k * ranks * upb <= kTileUnits
    uint32_t upb;              // units per block
    uint32_t inner, pj;        // the moving dimension (1, 1: same-rank copies)
    FastDiv d_upb, d_row, d_plane, d_inner, d_pj;   // upb; k_rows * upb; ranks * upb
};

__device__ __forceinline__ void fetch_now(const StagedRoundArgs &a) {
    asm volatile("" ::"s"(a.entries), "s"(a.map.n_tiles), "s"(a.map.run_log2), "s"(a.map.per_xcd), "s"(a.p), "s"(a.k),
                 "s"(a.k_rows), "s"(a.ranks), "s"(a.upb), "s"(a.inner), "s"(a.pj));
    fetch_now(a.d_upb);
    fetch_now(a.d_row);
    fetch_now(a.d_plane);
    fetch_now(a.d_inner);
    fetch_now(a.d_pj);
}

template <typename V, bool NTL, uint32_t UPL>
__global__ __launch_bounds__(kThreads) void staged_round_kernel(const StagedRoundArgs a) {
    fetch_now(a);
    __shared__ DevEntry lds[kLdsEntries];
    extern __shared__ __align__(16) unsigned char tile_bytes[];
    V *tile = (V *)tile_bytes;
    typedef typename Unaligned<V>::type UV;
    typedef const UV __attribute__((address_space(1))) *src_ptr;
    typedef UV __attribute__((address_space(1))) *dst_ptr;
    uint32_t tile_id;
    if (!tile_of_block(a.map, tile_id)) return;          // (before anything is loaded: the grid is padded)
    const EntryTable<true> table(a.entries, a.k, lds);
    const uint32_t R0 = tile_id * a.ranks;
    const uint32_t n = a.p - R0 < a.ranks ? a.p - R0 : a.ranks;
    const uint32_t plane = a.ranks * a.upb, pitch = plane + 1u;      // padded planes: the strided LDS writes spread over the banks
    const uint32_t n_rows = a.k_rows * plane, n_all = a.k * plane;
    V regs[UPL];
    uint32_t at[UPL];                          // where in the tile the unit goes; ~0: no unit
#pragma unroll
    for (uint32_t it = 0; it < UPL; ++it) {
        const uint32_t q = threadIdx.x + it * (uint32_t)kThreads;
        uint32_t e, r, c, rem;
        if (q < n_rows) {                                // (rank, entry, unit) over the rank-major sources
            fast_divmod(q, a.d_row, r, rem);
            fast_divmod(rem, a.d_upb, e, c);
        } else {                                         // (entry, rank, unit) over the slot-major sources
            fast_divmod(q - n_rows, a.d_plane, e, rem);
            fast_divmod(rem, a.d_upb, r, c);
            e += a.k_rows;
        }
        // a lane with no unit loads the tile's first unit instead and drops it: the eight loads stay
        // straight-line code, all in flight together
        const bool has_unit = q < n_all && r < n;
        e = has_unit ? e : 0u;
        r = has_unit ? r : 0u;
        c = has_unit ? c : 0u;
        const DevEntry en = table[e];
        const src_ptr sp = (src_ptr)(block_address(en.src, R0 + r, en.src_stride) + (uint64_t)c * sizeof(V));
        if constexpr (NTL && sizeof(V) == 16) regs[it] = __builtin_nontemporal_load(sp);
        else regs[it] = *sp;
        at[it] = has_unit ? e * pitch + r * a.upb + c : ~0u;
    }
#pragma unroll
    for (uint32_t it = 0; it < UPL; ++it)
        if (at[it] != ~0u) tile[at[it]] = regs[it];
    __syncthreads();
#pragma unroll
    for (uint32_t it = 0; it < UPL; ++it) {    // (entry, rank, unit): dense runs of every plane
        const uint32_t q = threadIdx.x + it * (uint32_t)kThreads;
        uint32_t e, r, c, rem;
        fast_divmod(q, a.d_plane, e, rem);
        fast_divmod(rem, a.d_upb, r, c);
        if (q < n_all && r < n) {
            const DevEntry en = table[e];
            // the tile's ranks are source ranks S: the block goes to the rank `shift` steps on
            const uint32_t S = R0 + r;
            const uint32_t qq = fast_div(S, a.d_inner);
            const uint32_t sj = qq - fast_div(qq, a.d_pj) * a.pj;
            uint32_t R = S + en.shift * a.inner;
            R -= sj + en.shift >= a.pj ? a.pj * a.inner : 0u;
            const dst_ptr dp = (dst_ptr)(block_address(en.dst, R, en.dst_stride) + (uint64_t)c * sizeof(V));
            if constexpr (sizeof(V) == 16) __builtin_nontemporal_store(tile[e * pitch + rem], dp);
            else *dp = tile[e * pitch + rem];
        }
    }
}

// Last launch of the staged schedule: entry i brings receive block i of every rank from where its
// last hop starts (a plane of the workspace or the send buffer), along the entry's own dimension.
// A workgroup takes `ranks` consecutive ranks: it reads their blocks in the order that suits the
// sources (as the rounds above do) into an LDS tile, one padded plane per receive block so that
// the strided LDS accesses spread over the banks, and writes the tile out in row order as one
// dense run of ranks * s * m bytes: small blocks are written as whole receive rows.
struct alignas(16) DeliverEntry {
    uint64_t src;          // address of rank 0's source block
    uint32_t src_stride;   // bytes between consecutive ranks in the source
    uint32_t slot;         // receive block i
    uint32_t shift, pj;    // residue v along the entry's dimension (0: same rank); that dimension's size
    uint32_t back, wrap;   // v * inner_j; p_j * inner_j
    FastDiv d_inner, d_pj;
};
static_assert(sizeof(DeliverEntry) == 64, "four 16-byte words per entry");

struct DeliverArgs {
    const DeliverEntry *entries;   // the first k_rows entries read a rank-major buffer
    uint64_t dst;                  // rank 0's receive row; rows of s blocks, back to back
    TileMap map;
    uint32_t p, s, k_rows;
    uint32_t ranks;                // ranks per workgroup: s * ranks * upb <= UPL * kThreads
    uint32_t upb;                  // units per block
    FastDiv d_upb, d_rows, d_plane, d_row;    // upb; k_rows * upb; ranks * upb; s * upb
};

__device__ __forceinline__ void fetch_now(const DeliverArgs &a) {
    asm volatile("" ::"s"(a.entries), "s"(a.dst), "s"(a.map.n_tiles), "s"(a.map.run_log2), "s"(a.map.per_xcd), "s"(a.p),
                 "s"(a.s), "s"(a.k_rows), "s"(a.ranks), "s"(a.upb));
    fetch_now(a.d_upb);
    fetch_now(a.d_rows);
    fetch_now(a.d_plane);
    fetch_now(a.d_row);
}

template <typename V, bool NTL, uint32_t UPL>
__global__ __launch_bounds__(kThreads) void deliver_kernel(const DeliverArgs a) {
    fetch_now(a);
    __shared__ DeliverEntry lds[kLdsEntries];
    extern __shared__ __align__(16) unsigned char tile_bytes[];
    V *tile = (V *)tile_bytes;
    typedef typename Unaligned<V>::type UV;
    typedef const UV __attribute__((address_space(1))) *src_ptr;
    typedef UV __attribute__((address_space(1))) *dst_ptr;
    uint32_t tile_id;
    if (!tile_of_block(a.map, tile_id)) return;          // (before anything is loaded: the grid is padded)
    for (uint32_t w = threadIdx.x; w < a.s * 4u; w += kThreads) ((vec16_t *)lds)[w] = ((const vec16_t *)a.entries)[w];
    __syncthreads();
    const uint32_t R0 = tile_id * a.ranks;
    const uint32_t n = a.p - R0 < a.ranks ? a.p - R0 : a.ranks;
    const uint32_t plane = a.ranks * a.upb, pitch = plane + 1u;
    const uint32_t n_rows = a.k_rows * plane, n_all = a.s * plane;
    V regs[UPL];
    uint32_t at[UPL];                                    // where in the tile the unit goes; ~0: no unit
#pragma unroll
    for (uint32_t it = 0; it < UPL; ++it) {
        const uint32_t q = threadIdx.x + it * (uint32_t)kThreads;
        uint32_t e, r, c, rem;
        if (q < n_rows) {                                // (rank, entry, unit) over the rank-major sources
            fast_divmod(q, a.d_rows, r, rem);
            fast_divmod(rem, a.d_upb, e, c);
        } else {                                         // (entry, rank, unit) over the planes
            fast_divmod(q - n_rows, a.d_plane, e, rem);
            fast_divmod(rem, a.d_upb, r, c);
            e += a.k_rows;
        }
        // a lane with no unit loads the tile's first unit instead and drops it
        const bool has_unit = q < n_all && r < n;
        e = has_unit ? e : 0u;
        r = has_unit ? r : 0u;
        c = has_unit ? c : 0u;
        const DeliverEntry &en = lds[e];
        const uint32_t R = R0 + r;
        const uint32_t qq = fast_div(R, en.d_inner);
        const uint32_t rj = qq - fast_div(qq, en.d_pj) * en.pj;
        const uint32_t srcR = R - en.back + (rj < en.shift ? en.wrap : 0u);
        const src_ptr sp = (src_ptr)(block_address(en.src, srcR, en.src_stride) + (uint64_t)c * sizeof(V));
        if constexpr (NTL && sizeof(V) == 16) regs[it] = __builtin_nontemporal_load(sp);
        else regs[it] = *sp;
        at[it] = has_unit ? en.slot * pitch + r * a.upb + c : ~0u;
    }
#pragma unroll
    for (uint32_t it = 0; it < UPL; ++it)
        if (at[it] != ~0u) tile[at[it]] = regs[it];
    __syncthreads();
    const uint64_t out = a.dst + (uint64_t)R0 * a.s * a.upb * sizeof(V);
#pragma unroll
    for (uint32_t it = 0; it < UPL; ++it) {              // (rank, block, unit): the receive rows, back to back
        const uint32_t q = threadIdx.x + it * (uint32_t)kThreads;
        uint32_t i, r, c, rem;
        fast_divmod(q, a.d_row, r, rem);
        fast_divmod(rem, a.d_upb, i, c);
        if (r < n) {
            const dst_ptr dp = (dst_ptr)(out + (uint64_t)q * sizeof(V));
            if constexpr (sizeof(V) == 16) __builtin_nontemporal_store(tile[i * pitch + r * a.upb + c], dp);
            else *dp = tile[i * pitch + r * a.upb + c];
        }
    }
}

// Plain streaming copy with the same access shape: the measured ceiling.
template <typename V>
__global__ __launch_bounds__(kThreads) void copy_kernel(const V *__restrict__ src, V *__restrict__ dst,
                                                        uint64_t n_units) {
    const uint64_t u = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (u < n_units) __builtin_nontemporal_store(__builtin_nontemporal_load(src + u), dst + u);
}

// Writes up to kStoreWords 32-bit words, carried in the kernel's own arguments, to device
// memory: how a table of block index maps reaches the device when the host may neither
// allocate nor copy (the launch itself is the transfer, and it is ordered by the stream).
constexpr uint32_t kStoreWords = 768;
struct TableChunk {
    uint32_t *dst;
    uint32_t n;            // words to write, at most kStoreWords
    uint32_t reserved;
    uint32_t words[kStoreWords];
};

__global__ __launch_bounds__(kThreads) void table_store_kernel(const TableChunk c) {
    const uint32_t i = blockIdx.x * (uint32_t)kThreads + threadIdx.x;
    if (i < c.n) c.dst[i] = c.words[i];
}

}  // namespace iso
