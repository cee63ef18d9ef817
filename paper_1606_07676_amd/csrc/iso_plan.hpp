// Host-side schedule builder: torus + neighbourhood -> per-launch block index
// maps.  Pure C++ (no HIP); everything here is O(s d) integer work.
#pragma once

#include <cstdint>
#include <vector>

#include "iso.h"

namespace iso {

struct Comm {
    int d = 0;
    int s = 0;
    int64_t p = 1;
    std::vector<int32_t> dims;       // p_j
    std::vector<int64_t> inner;      // prod_{l>j} p_l : rank stride of dimension j
    std::vector<int32_t> raw;        // s*d offsets as given
    std::vector<int32_t> can;        // s*d effective coordinates: residue in [0, p_j) where the
                                     // dimension is periodic, the raw signed value where it is not
    std::vector<uint8_t> periodic;   // d flags
    bool mesh = false;               // some dimension does not wrap
    std::vector<std::vector<int32_t>> values;  // per dimension: sorted distinct non-zero residues

    int32_t c(int i, int j) const { return can[(size_t)i * d + j]; }
    int nnz(int i) const;
    int rounds() const;
};

struct Round {
    int kind = ISO_ROUND_SHIFT;
    int dim = -1;
    std::vector<iso_plan_entry_t> entries;
};

struct Plan {
    int op = ISO_OP_ALLTOALL;
    int algorithm = ISO_ALG_COMBINED;
    int work_slots = 0;
    std::vector<int32_t> dim_order;
    std::vector<Round> rounds;
    Comm comm;                       // own copy: a plan outlives its communicator

    int64_t entries() const;
};

// Validates and canonicalises; returns ISO_SUCCESS or ISO_ERR_*.
// `periodic` may be null (all dimensions wrap).
int build_comm(int d, const int32_t *dims, const int32_t *periodic, int s, const int32_t *rel, Comm &out);

// Order in which the allgather trie visits the dimensions: the identity order
// unless the fewest-distinct-values-first order moves strictly fewer blocks.
std::vector<int32_t> allgather_dim_order(const Comm &c, int64_t *moves_out);

int build_plan(const Comm &c, int op, int algorithm, Plan &out);

}  // namespace iso
