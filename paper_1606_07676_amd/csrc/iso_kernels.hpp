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
// ordered (rank, entry, chunk-in-block), chunk fastest.  Consecutive lanes
// therefore touch consecutive 16-byte pieces of one block, then the next block
// of the same rank: every wavefront load/store covers whole blocks.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "iso.h"
#include "iso_fastdiv.hpp"

namespace iso {

constexpr int kThreads = 256;

struct alignas(16) DevEntry {
    uint64_t src;          // address of rank 0's source block
    uint64_t dst;          // address of rank 0's destination block
    uint64_t src_stride;   // bytes between consecutive ranks in the source buffer
    uint64_t dst_stride;
    uint32_t shift;        // SHIFT rounds: residue v; VECTOR rounds: neighbour index
    uint32_t pad[3];
};

struct ShiftArgs {
    const DevEntry *entries;
    uint32_t total;        // units in this launch = p * k * chunks
    uint32_t n_blocks;     // workgroups that carry work
    uint32_t blocks_per_xcd;
    uint32_t inner;        // rank stride of the shifted dimension
    uint32_t pj;           // its size
    FastDiv d_chunks, d_k, d_inner, d_pj;
};

struct VectorArgs {
    const DevEntry *entries;
    const uint32_t *offsets;   // [s][d] residues
    uint32_t total;
    uint32_t n_blocks;
    uint32_t blocks_per_xcd;
    int32_t d;
    FastDiv d_chunks, d_k;
    FastDiv d_dims[ISO_MAX_DIMS];
    uint32_t inner[ISO_MAX_DIMS];
};

typedef uint32_t vec16_t __attribute__((ext_vector_type(4)));
typedef uint32_t vec8_t __attribute__((ext_vector_type(2)));

template <typename V, bool NT>
__device__ __forceinline__ V load_unit(const V *p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <typename V, bool NT>
__device__ __forceinline__ void store_unit(V *p, V v) {
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Workgroups are handed to the 8 XCDs round-robin.  With XCD remapping, XCD x
// works on the x-th contiguous eighth of the launch, so that neighbouring ranks'
// blocks (which can share cache lines and DRAM pages) go through one L2.
template <bool XCD>
__device__ __forceinline__ bool logical_block(uint32_t n_blocks, uint32_t blocks_per_xcd, uint32_t &bid) {
    bid = blockIdx.x;
    if constexpr (XCD) {
        const uint32_t y = bid >> 3;
        bid = (bid & 7u) * blocks_per_xcd + y;
        if (y >= blocks_per_xcd) return false;
    }
    return bid < n_blocks;
}

template <typename V, int UNROLL, bool NT, bool XCD>
__global__ __launch_bounds__(kThreads) void shift_round_kernel(const ShiftArgs a) {
    uint32_t bid;
    if (!logical_block<XCD>(a.n_blocks, a.blocks_per_xcd, bid)) return;
    const uint32_t base = bid * (uint32_t)(kThreads * UNROLL) + threadIdx.x;
    V val[UNROLL];
    V *dst[UNROLL];
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) {
        const uint32_t u = base + (uint32_t)i * kThreads;
        dst[i] = nullptr;
        if (u < a.total) {
            uint32_t t, ch, R, e, q, rj;
            fast_divmod(u, a.d_chunks, t, ch);
            fast_divmod(t, a.d_k, R, e);
            q = fast_div(R, a.d_inner);
            rj = q - fast_div(q, a.d_pj) * a.pj;
            const DevEntry en = a.entries[e];
            // v steps back along the dimension, with wrap-around
            const int64_t back = rj >= en.shift ? -(int64_t)en.shift : (int64_t)(a.pj - en.shift);
            const uint64_t srcR = (uint64_t)((int64_t)R + back * (int64_t)a.inner);
            const V *sp = reinterpret_cast<const V *>(en.src + srcR * en.src_stride) + ch;
            dst[i] = reinterpret_cast<V *>(en.dst + (uint64_t)R * en.dst_stride) + ch;
            val[i] = load_unit<V, NT>(sp);
        }
    }
#pragma unroll
    for (int i = 0; i < UNROLL; ++i)
        if (dst[i]) store_unit<V, NT>(dst[i], val[i]);
}

template <typename V, int UNROLL, bool NT, bool XCD>
__global__ __launch_bounds__(kThreads) void vector_round_kernel(const VectorArgs a) {
    uint32_t bid;
    if (!logical_block<XCD>(a.n_blocks, a.blocks_per_xcd, bid)) return;
    const uint32_t base = bid * (uint32_t)(kThreads * UNROLL) + threadIdx.x;
    V val[UNROLL];
    V *dst[UNROLL];
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) {
        const uint32_t u = base + (uint32_t)i * kThreads;
        dst[i] = nullptr;
        if (u < a.total) {
            uint32_t t, ch, R, e;
            fast_divmod(u, a.d_chunks, t, ch);
            fast_divmod(t, a.d_k, R, e);
            const DevEntry en = a.entries[e];
            const uint32_t *c = a.offsets + (size_t)en.shift * a.d;
            int64_t srcR = R;
            uint32_t rem = R;
            for (int j = a.d - 1; j >= 0; --j) {
                uint32_t q, rj;
                fast_divmod(rem, a.d_dims[j], q, rj);
                rem = q;
                const uint32_t cj = c[j];
                const int64_t back = rj >= cj ? -(int64_t)cj : (int64_t)(a.d_dims[j].div - cj);
                srcR += back * (int64_t)a.inner[j];
            }
            const V *sp = reinterpret_cast<const V *>(en.src + (uint64_t)srcR * en.src_stride) + ch;
            dst[i] = reinterpret_cast<V *>(en.dst + (uint64_t)R * en.dst_stride) + ch;
            val[i] = load_unit<V, NT>(sp);
        }
    }
#pragma unroll
    for (int i = 0; i < UNROLL; ++i)
        if (dst[i]) store_unit<V, NT>(dst[i], val[i]);
}

// Plain streaming copy with the same access shape: the measured ceiling.
template <typename V, int UNROLL, bool NT>
__global__ __launch_bounds__(kThreads) void copy_kernel(const V *__restrict__ src, V *__restrict__ dst,
                                                        uint64_t n_units) {
    const uint64_t base = (uint64_t)blockIdx.x * (kThreads * UNROLL) + threadIdx.x;
    V val[UNROLL];
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) {
        const uint64_t u = base + (uint64_t)i * kThreads;
        if (u < n_units) val[i] = load_unit<V, NT>(src + u);
    }
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) {
        const uint64_t u = base + (uint64_t)i * kThreads;
        if (u < n_units) store_unit<V, NT>(dst + u, val[i]);
    }
}

}  // namespace iso
