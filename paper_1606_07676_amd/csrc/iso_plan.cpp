// Schedule builder for isomorphic sparse collectives (host only).
//
// All-to-all: Algorithm 1's alternating-buffer rule, applied either to the
// torus-direct schedule of Section 5 (a block makes one hop per non-zero
// coordinate; each dimension has one round per distinct non-zero coordinate
// value) or to the one-ported torus schedule of Section 3.1 (one hop per unit
// of coordinate; positive steps, then negative steps, per dimension).
// Allgather: the prefix trie of Section 3.2, routed the same two ways.
// S-exchange: the straightforward algorithm of Section 3's first listing.
#include "iso_plan.hpp"

#include <algorithm>
#include <cstdlib>
#include <functional>
#include <numeric>
#include <queue>

namespace iso {

constexpr int64_t kMaxOneHopRounds = 1 << 16;

int Comm::nnz(int i) const {
    int n = 0;
    for (int j = 0; j < d; ++j) n += c(i, j) != 0;
    return n;
}

int Comm::rounds() const {
    size_t n = 0;
    for (const auto &v : values) n += v.size();
    return (int)n;
}

int64_t Plan::entries() const {
    int64_t n = 0;
    for (const auto &r : rounds) n += (int64_t)r.entries.size();
    return n;
}

int build_comm(int d, const int32_t *dims, const int32_t *periodic, int s, const int32_t *rel, Comm &out) {
    if (d < 1 || d > ISO_MAX_DIMS || !dims || s < 0 || (s > 0 && !rel)) return ISO_ERR_ARG;
    Comm c;
    c.d = d;
    c.s = s;
    c.dims.assign(dims, dims + d);
    c.p = 1;
    for (int j = 0; j < d; ++j) {
        if (dims[j] < 1) return ISO_ERR_ARG;
        c.p *= dims[j];
        if (c.p >= (int64_t(1) << 31)) return ISO_ERR_TOO_LARGE;
    }
    c.inner.assign(d, 1);
    for (int j = d - 2; j >= 0; --j) c.inner[j] = c.inner[j + 1] * dims[j + 1];
    c.periodic.assign(d, 1);
    for (int j = 0; j < d && periodic; ++j) {
        c.periodic[j] = periodic[j] != 0;
        c.mesh = c.mesh || !c.periodic[j];
    }
    c.raw.assign(rel, rel + (size_t)s * d);
    c.can.resize((size_t)s * d);
    c.values.assign(d, {});
    for (int i = 0; i < s; ++i)
        for (int j = 0; j < d; ++j) {
            int64_t r = rel[(size_t)i * d + j];
            if (c.periodic[j]) {
                r %= dims[j];
                if (r < 0) r += dims[j];
            }
            c.can[(size_t)i * d + j] = (int32_t)r;
            if (r) c.values[j].push_back((int32_t)r);
        }
    for (auto &v : c.values) {
        std::sort(v.begin(), v.end());
        v.erase(std::unique(v.begin(), v.end()), v.end());
    }
    out = std::move(c);
    return ISO_SUCCESS;
}

namespace {

iso_plan_entry_t mk(int sb, int ss, int db, int ds, int shift, int nb) {
    iso_plan_entry_t e;
    e.src_buf = sb; e.src_slot = ss; e.dst_buf = db; e.dst_slot = ds;
    e.shift = shift; e.neighbor = nb;
    e.ref = nb;
    e.dim = -1;
    return e;
}

// Coordinates as the schedule sees them: residues (torus-direct) or the raw signed
// values (one-hop, where |c| is the number of hops and the sign the direction).
struct Coords {
    const Comm &c;
    bool raw;
    int32_t at(int i, int j) const { return raw ? c.raw[(size_t)i * c.d + j] : c.c(i, j); }
    bool zero(int i) const {
        for (int j = 0; j < c.d; ++j)
            if (at(i, j)) return false;
        return true;
    }
};

// residue that means "one step back" (direction +1) or "one step forward" (-1)
int32_t unit_shift(const Comm &c, int j, int sign) {
    const int32_t pj = c.dims[j];
    return sign > 0 ? 1 % pj : (pj - 1) % pj;
}

bool by_dst(const iso_plan_entry_t &a, const iso_plan_entry_t &b) {
    return a.dst_buf != b.dst_buf ? a.dst_buf < b.dst_buf : a.dst_slot < b.dst_slot;
}

// ---------------------------------------------------------------------------
// all-to-all, message-combining
// ---------------------------------------------------------------------------
struct AlltoallState {
    std::vector<int> hops, where, where_slot, wslot, wslot2;
    bool mesh = false;
    // one hop of block i: parity rule of Algorithm 1
    iso_plan_entry_t hop(int i, int shift) {
        // received into the receive buffer when an odd number of hops remains,
        // so that the last hop (one remaining) always lands there.  On a mesh the
        // receive buffer takes only that last hop (a block in transit must not
        // overwrite a receive block that is to stay untouched): earlier odd hops
        // go to a second workspace slot.
        int dst = (hops[i] % 2 == 0) ? ISO_BUF_WORK : ISO_BUF_RECV;
        int dslot = dst == ISO_BUF_WORK ? wslot[i] : i;
        if (mesh && dst == ISO_BUF_RECV && hops[i] > 1) {
            dst = ISO_BUF_WORK;
            dslot = wslot2[i];
        }
        iso_plan_entry_t e = mk(where[i], where_slot[i], dst, dslot, shift, i);
        where[i] = dst;
        where_slot[i] = dslot;
        --hops[i];
        return e;
    }
};

void alltoall_prologue(const Comm &c, const Coords &co, AlltoallState &st, Plan &pl) {
    const int s = c.s;
    st.hops.assign(s, 0);
    st.where.assign(s, ISO_BUF_SEND);
    st.where_slot.resize(s);
    std::iota(st.where_slot.begin(), st.where_slot.end(), 0);
    st.wslot.assign(s, -1);
    st.wslot2.assign(s, -1);
    st.mesh = c.mesh;
    int nwork = 0;
    Round self;
    self.kind = ISO_ROUND_SELF;
    for (int i = 0; i < s; ++i) {
        for (int j = 0; j < c.d; ++j) st.hops[i] += co.raw ? std::abs(co.at(i, j)) : (co.at(i, j) != 0);
        if (st.hops[i] >= 2) st.wslot[i] = nwork++;     // only these ever sit in the intermediate buffer
        if (c.mesh && st.hops[i] >= 3) st.wslot2[i] = nwork++;
        if (st.hops[i] == 0) self.entries.push_back(mk(ISO_BUF_SEND, i, ISO_BUF_RECV, i, 0, i));
    }
    pl.work_slots = nwork;
    if (!self.entries.empty()) pl.rounds.push_back(std::move(self));
}

void plan_alltoall_combined(const Comm &c, bool by_dim, Plan &pl) {
    const Coords co{c, false};
    AlltoallState st;
    alltoall_prologue(c, co, st, pl);
    for (int j = 0; j < c.d; ++j) {
        Round dim_round;
        dim_round.dim = j;
        for (int32_t v : c.values[j]) {
            Round r;
            r.dim = j;
            for (int i = 0; i < c.s; ++i)
                if (c.c(i, j) == v) r.entries.push_back(st.hop(i, v));
            if (by_dim)
                dim_round.entries.insert(dim_round.entries.end(), r.entries.begin(), r.entries.end());
            else
                pl.rounds.push_back(std::move(r));
        }
        if (by_dim && !dim_round.entries.empty()) {
            std::stable_sort(dim_round.entries.begin(), dim_round.entries.end(),
                             [](const iso_plan_entry_t &a, const iso_plan_entry_t &b) {
                                 return a.neighbor < b.neighbor;
                             });
            pl.rounds.push_back(std::move(dim_round));
        }
    }
}

void plan_alltoall_onehop(const Comm &c, Plan &pl) {
    const Coords co{c, true};
    AlltoallState st;
    alltoall_prologue(c, co, st, pl);
    for (int j = 0; j < c.d; ++j)
        for (int sign = +1; sign >= -1; sign -= 2) {            // positive steps, then negative
            int32_t most = 0;
            for (int i = 0; i < c.s; ++i) most = std::max(most, sign * co.at(i, j));
            for (int32_t h = 0; h < most; ++h) {
                Round r;
                r.dim = j;
                for (int i = 0; i < c.s; ++i)
                    if (sign * co.at(i, j) > h) r.entries.push_back(st.hop(i, unit_shift(c, j, sign)));
                pl.rounds.push_back(std::move(r));
            }
        }
}

// ---------------------------------------------------------------------------
// allgather, message-combining along the prefix trie
// ---------------------------------------------------------------------------
struct Node {
    int parent;        // node index, -1 for the root
    int level;         // index into the dimension order; root: -1
    int32_t value;     // coordinate on the edge from the parent
    int first, last;   // range [first, last) of the sorted neighbour list below this node
    int store;         // nearest node on the path to the root (incl. self) that holds a copy
    int buf, slot;     // where that copy sits (stored nodes only; root: send block)
    int tmp_slot;      // one-hop, |value| >= 2: second workspace slot the block alternates through
    int last_read;     // last level at which a child reads this copy
    std::vector<int> terminals;  // neighbours equal to this prefix padded with zeros
};

void build_trie(const Coords &co, const std::vector<int32_t> &order, std::vector<int> &sorted,
                std::vector<Node> &nodes) {
    const int s = co.c.s, d = co.c.d;
    sorted.resize(s);
    std::iota(sorted.begin(), sorted.end(), 0);
    // zero first, then by value: neighbours that end at a node head its range
    auto key = [](int32_t v) { return std::make_pair(v != 0, v); };
    std::stable_sort(sorted.begin(), sorted.end(), [&](int a, int b) {
        for (int t = 0; t < d; ++t) {
            int32_t x = co.at(a, order[t]), y = co.at(b, order[t]);
            if (x != y) return key(x) < key(y);
        }
        return false;
    });
    nodes.clear();
    Node root{};
    root.parent = -1; root.level = -1; root.value = 0; root.first = 0; root.last = s;
    root.store = 0; root.buf = ISO_BUF_SEND; root.slot = 0; root.tmp_slot = -1; root.last_read = -1;
    nodes.push_back(root);
    size_t level_begin = 0, level_end = 1;
    for (int t = 0; t < d; ++t) {
        const int j = order[t];
        for (size_t n = level_begin; n < level_end; ++n) {
            int a = nodes[n].first;
            const int end = nodes[n].last;
            while (a < end) {
                const int32_t v = co.at(sorted[a], j);
                int b = a;
                while (b < end && co.at(sorted[b], j) == v) ++b;
                Node ch{};
                ch.parent = (int)n; ch.level = t; ch.value = v; ch.first = a; ch.last = b;
                ch.buf = -1; ch.slot = -1; ch.tmp_slot = -1; ch.last_read = -1;
                ch.store = v ? (int)nodes.size() : nodes[n].store;
                if (v) {
                    // neighbours that end here: all later coordinates zero; they sort first
                    for (int q = a; q < b; ++q) {
                        bool rest_zero = true;
                        for (int u = t + 1; u < d && rest_zero; ++u)
                            rest_zero = co.at(sorted[q], order[u]) == 0;
                        if (!rest_zero) break;
                        ch.terminals.push_back(sorted[q]);
                    }
                }
                nodes.push_back(std::move(ch));
                a = b;
            }
        }
        level_begin = level_end;
        level_end = nodes.size();
    }
}

// block-moves per rank: one per hop of every stored node, plus one per repeated neighbour
int64_t trie_moves(const std::vector<Node> &nodes, bool per_hop) {
    int64_t n = 0;
    for (const Node &nd : nodes)
        if (nd.level >= 0 && nd.value) {
            n += per_hop ? std::abs(nd.value) : 1;
            if (nd.terminals.size() > 1) n += (int64_t)nd.terminals.size() - 1;
        }
    return n;
}

std::vector<int32_t> pick_dim_order(const Coords &co, int64_t *moves_out) {
    const Comm &c = co.c;
    const int d = c.d;
    std::vector<int32_t> ident(d), heur(d);
    std::iota(ident.begin(), ident.end(), 0);
    heur = ident;
    // candidate: dimensions with few distinct values first, so that prefixes are
    // shared by many neighbours (Section 3.2's remark on visiting order)
    std::vector<int> distinct(d), maxmult(d, 0);
    for (int j = 0; j < d; ++j) {
        std::vector<int32_t> col(c.s);
        for (int i = 0; i < c.s; ++i) col[i] = co.at(i, j);
        std::sort(col.begin(), col.end());
        int run = 0;
        distinct[j] = 0;
        for (int i = 0; i < c.s; ++i) {
            if (i == 0 || col[i] != col[i - 1]) { ++distinct[j]; run = 0; }
            maxmult[j] = std::max(maxmult[j], ++run);
        }
    }
    std::stable_sort(heur.begin(), heur.end(), [&](int a, int b) {
        if (distinct[a] != distinct[b]) return distinct[a] < distinct[b];
        return maxmult[a] > maxmult[b];
    });
    std::vector<int> sorted;
    std::vector<Node> nodes;
    build_trie(co, ident, sorted, nodes);
    const int64_t mi = trie_moves(nodes, co.raw);
    int64_t mh = mi;
    if (heur != ident) {
        build_trie(co, heur, sorted, nodes);
        mh = trie_moves(nodes, co.raw);
    }
    if (mh < mi) {
        if (moves_out) *moves_out = mh;
        return heur;
    }
    if (moves_out) *moves_out = mi;
    return ident;
}

// Where every stored node keeps its copy: the receive slot of a neighbour that
// ends at the node, else a workspace slot; workspace slots are handed out again
// once the level of their last reader has passed.  One-hop nodes with two or
// more hops also get a second slot for the duration of their own level.
int assign_storage(std::vector<Node> &nodes, int d, bool per_hop) {
    for (size_t n = 1; n < nodes.size(); ++n)
        if (nodes[n].value) {
            Node &src = nodes[nodes[nodes[n].parent].store];
            src.last_read = std::max(src.last_read, nodes[n].level);
        }
    std::priority_queue<int, std::vector<int>, std::greater<int>> free_slots;
    std::vector<std::pair<int, int>> live;   // (last level that reads it, slot)
    int nwork = 0;
    auto take = [&](int last_read) {
        int slot;
        if (free_slots.empty()) {
            slot = nwork++;
        } else {
            slot = free_slots.top();
            free_slots.pop();
        }
        live.emplace_back(last_read, slot);
        return slot;
    };
    size_t n = 1;
    for (int t = 0; t < d; ++t) {
        for (size_t q = 0; q < live.size();) {
            if (live[q].first < t) {
                free_slots.push(live[q].second);
                live[q] = live.back();
                live.pop_back();
            } else {
                ++q;
            }
        }
        for (; n < nodes.size() && nodes[n].level == t; ++n) {
            Node &nd = nodes[n];
            if (!nd.value) continue;
            if (!nd.terminals.empty()) {
                nd.buf = ISO_BUF_RECV;
                nd.slot = nd.terminals[0];
            } else {
                nd.buf = ISO_BUF_WORK;
                nd.slot = take(nd.last_read);
            }
            if (per_hop && std::abs(nd.value) >= 2) nd.tmp_slot = take(t);
        }
    }
    return nwork;
}

void allgather_self_round(const Coords &co, Plan &pl) {
    Round self;
    self.kind = ISO_ROUND_SELF;
    for (int i = 0; i < co.c.s; ++i)
        if (co.zero(i)) self.entries.push_back(mk(ISO_BUF_SEND, 0, ISO_BUF_RECV, i, 0, i));
    if (!self.entries.empty()) pl.rounds.push_back(std::move(self));
}

void plan_allgather_combined(const Comm &c, bool by_dim, Plan &pl) {
    const Coords co{c, false};
    const int d = c.d;
    pl.dim_order = pick_dim_order(co, nullptr);
    std::vector<int> sorted;
    std::vector<Node> nodes;
    build_trie(co, pl.dim_order, sorted, nodes);
    allgather_self_round(co, pl);
    pl.work_slots = assign_storage(nodes, d, false);

    size_t n = 1;
    for (int t = 0; t < d; ++t) {
        const int j = pl.dim_order[t];
        const size_t lvl_begin = n;
        while (n < nodes.size() && nodes[n].level == t) ++n;
        Round dim_round;
        dim_round.dim = j;
        for (int32_t v : c.values[j]) {
            Round r;
            r.dim = j;
            for (size_t q = lvl_begin; q < n; ++q) {
                const Node &nd = nodes[q];
                if (nd.value != v) continue;
                const Node &src = nodes[nodes[nd.parent].store];
                if (nd.terminals.empty()) {
                    r.entries.push_back(mk(src.buf, src.slot, nd.buf, nd.slot, v, -1));
                    r.entries.back().ref = sorted[(size_t)nd.first];
                } else {
                    for (int i : nd.terminals)       // repeated offsets: one copy each
                        r.entries.push_back(mk(src.buf, src.slot, ISO_BUF_RECV, i, v, i));
                }
            }
            std::stable_sort(r.entries.begin(), r.entries.end(), by_dst);
            if (by_dim)
                dim_round.entries.insert(dim_round.entries.end(), r.entries.begin(), r.entries.end());
            else if (!r.entries.empty())
                pl.rounds.push_back(std::move(r));
        }
        if (by_dim && !dim_round.entries.empty()) {
            std::stable_sort(dim_round.entries.begin(), dim_round.entries.end(), by_dst);
            pl.rounds.push_back(std::move(dim_round));
        }
    }
}

void plan_allgather_onehop(const Comm &c, Plan &pl) {
    const Coords co{c, true};
    const int d = c.d;
    pl.dim_order = pick_dim_order(co, nullptr);
    std::vector<int> sorted;
    std::vector<Node> nodes;
    build_trie(co, pl.dim_order, sorted, nodes);
    allgather_self_round(co, pl);
    pl.work_slots = assign_storage(nodes, d, true);

    // where a node's block sits while it travels: parent's copy before the first hop
    std::vector<std::pair<int, int>> at(nodes.size());
    size_t n = 1;
    for (int t = 0; t < d; ++t) {
        const int j = pl.dim_order[t];
        const size_t lvl_begin = n;
        while (n < nodes.size() && nodes[n].level == t) ++n;
        for (size_t q = lvl_begin; q < n; ++q) {
            const Node &src = nodes[nodes[nodes[q].parent].store];
            at[q] = {src.buf, src.slot};
        }
        for (int sign = +1; sign >= -1; sign -= 2) {
            int32_t most = 0;
            for (size_t q = lvl_begin; q < n; ++q) most = std::max(most, sign * nodes[q].value);
            for (int32_t h = 0; h < most; ++h) {
                Round r;
                r.dim = j;
                const int32_t shift = unit_shift(c, j, sign);
                for (size_t q = lvl_begin; q < n; ++q) {
                    const Node &nd = nodes[q];
                    if (sign * nd.value <= h) continue;
                    const int32_t remaining = sign * nd.value - h;
                    // odd number of hops left: into the node's own place, else the spare slot
                    if (remaining == 1) {
                        if (nd.terminals.empty()) {
                            r.entries.push_back(mk(at[q].first, at[q].second, nd.buf, nd.slot, shift, -1));
                            r.entries.back().ref = sorted[(size_t)nd.first];
                        } else {
                            for (int i : nd.terminals)
                                r.entries.push_back(mk(at[q].first, at[q].second, ISO_BUF_RECV, i, shift, i));
                        }
                        at[q] = {nd.buf, nd.slot};
                    } else {
                        const std::pair<int, int> dst = remaining % 2 ? std::make_pair(nd.buf, nd.slot)
                                                                      : std::make_pair((int)ISO_BUF_WORK, nd.tmp_slot);
                        r.entries.push_back(mk(at[q].first, at[q].second, dst.first, dst.second, shift,
                                               nd.terminals.empty() ? -1 : nd.terminals[0]));
                        r.entries.back().ref = sorted[(size_t)nd.first];
                        at[q] = dst;
                    }
                }
                std::stable_sort(r.entries.begin(), r.entries.end(), by_dst);
                pl.rounds.push_back(std::move(r));
            }
        }
    }
}

// ---------------------------------------------------------------------------
// straightforward s-exchange
// ---------------------------------------------------------------------------
void plan_s_exchange(const Comm &c, int op, bool fused, Plan &pl) {
    Round all;
    all.kind = ISO_ROUND_VECTOR;
    for (int i = 0; i < c.s; ++i) {
        iso_plan_entry_t e = mk(ISO_BUF_SEND, op == ISO_OP_ALLTOALL ? i : 0, ISO_BUF_RECV, i, 0, i);
        if (fused) {
            all.entries.push_back(e);
        } else {
            Round r;
            r.kind = ISO_ROUND_VECTOR;
            r.entries.push_back(e);
            pl.rounds.push_back(std::move(r));
        }
    }
    if (fused && !all.entries.empty()) pl.rounds.push_back(std::move(all));
}

}  // namespace

std::vector<int32_t> allgather_dim_order(const Comm &c, int64_t *moves_out) {
    return pick_dim_order(Coords{c, false}, moves_out);
}

int build_plan(const Comm &c, int op, int algorithm, Plan &out) {
    if (op != ISO_OP_ALLTOALL && op != ISO_OP_ALLGATHER) return ISO_ERR_ARG;
    Plan pl;
    pl.op = op;
    pl.algorithm = algorithm;
    pl.comm = c;
    pl.dim_order.resize(c.d);
    std::iota(pl.dim_order.begin(), pl.dim_order.end(), 0);
    switch (algorithm) {
        case ISO_ALG_COMBINED:
        case ISO_ALG_COMBINED_BYDIM:
            if (op == ISO_OP_ALLTOALL)
                plan_alltoall_combined(c, algorithm == ISO_ALG_COMBINED_BYDIM, pl);
            else
                plan_allgather_combined(c, algorithm == ISO_ALG_COMBINED_BYDIM, pl);
            break;
        case ISO_ALG_COMBINED_STAGED: {
            // The message-combining schedule, regrouped so that the receive buffer is written only once, by
            // the last launch, a whole row at a time.  Every move keeps its source, distance and dimension:
            //  - a move into the receive buffer that is the last one for its block, whose block nobody
            //    reads afterwards and whose source stays as it is until the end, is taken out of its round
            //    and put into the last launch (kind DELIVER: every entry moves along its own dimension);
            //  - any other move into the receive buffer goes to a staging slot of the workspace instead
            //    (and reads of that block follow it there); if it was the block's last, the last launch
            //    copies the staging slot into the receive block.
            // Rounds left without entries disappear.  The workspace is one dense plane per slot, so all
            // rounds before the last write dense streams whatever the block size is.
            if (c.mesh) return ISO_ERR_ARG;      // on a mesh untouched receive blocks must keep their content
            // (built on the rounds of a dimension taken together, as ISO_ALG_COMBINED_BYDIM does: the pieces that
            // the + and - rounds of a dimension read from a send-buffer row share memory lines; 5 % at 16 bytes)
            if (op == ISO_OP_ALLTOALL)
                plan_alltoall_combined(c, true, pl);
            else
                plan_allgather_combined(c, true, pl);
            std::vector<Round> in = std::move(pl.rounds);
            pl.rounds.clear();
            const int n_in = (int)in.size();
            // last round that writes a (buffer, slot); last round that reads receive block i
            std::vector<int> last_write_recv((size_t)c.s, -1), last_read_recv((size_t)c.s, -1);
            std::vector<int> last_write_work((size_t)pl.work_slots, -1);
            for (int ri = 0; ri < n_in; ++ri)
                for (const iso_plan_entry_t &e : in[(size_t)ri].entries) {
                    if (e.dst_buf == ISO_BUF_RECV) last_write_recv[(size_t)e.dst_slot] = ri;
                    if (e.dst_buf == ISO_BUF_WORK) last_write_work[(size_t)e.dst_slot] = ri;
                    if (e.src_buf == ISO_BUF_RECV) last_read_recv[(size_t)e.src_slot] = ri;
                }
            std::vector<int> stage((size_t)c.s, -1);
            auto stage_of = [&](int i) {
                if (stage[(size_t)i] < 0) stage[(size_t)i] = pl.work_slots++;
                return stage[(size_t)i];
            };
            Round deliver;
            deliver.kind = ISO_ROUND_DELIVER;
            deliver.dim = -1;
            deliver.entries.resize((size_t)c.s);
            for (int ri = 0; ri < n_in; ++ri) {
                Round out;
                out.kind = in[(size_t)ri].kind;
                out.dim = in[(size_t)ri].dim;
                for (iso_plan_entry_t e : in[(size_t)ri].entries) {
                    const bool source_stays =
                        e.src_buf == ISO_BUF_SEND ||
                        (e.src_buf == ISO_BUF_WORK && last_write_work[(size_t)e.src_slot] < ri) ||
                        (e.src_buf == ISO_BUF_RECV && last_write_recv[(size_t)e.src_slot] < ri);
                    if (e.src_buf == ISO_BUF_RECV) { e.src_buf = ISO_BUF_WORK; e.src_slot = stage_of(e.src_slot); }
                    if (e.dst_buf != ISO_BUF_RECV) { out.entries.push_back(e); continue; }
                    const int i = e.dst_slot;
                    const bool last_for_block = last_write_recv[(size_t)i] == ri;
                    if (last_for_block && last_read_recv[(size_t)i] < ri && source_stays) {
                        e.dim = out.kind == ISO_ROUND_SHIFT ? out.dim : -1;
                        deliver.entries[(size_t)i] = e;
                        continue;
                    }
                    e.dst_buf = ISO_BUF_WORK;
                    e.dst_slot = stage_of(i);
                    out.entries.push_back(e);
                    if (last_for_block) {
                        iso_plan_entry_t cp{};
                        cp.src_buf = ISO_BUF_WORK; cp.src_slot = e.dst_slot;
                        cp.dst_buf = ISO_BUF_RECV; cp.dst_slot = i;
                        cp.shift = 0; cp.neighbor = i; cp.ref = i; cp.dim = -1;
                        deliver.entries[(size_t)i] = cp;
                    }
                }
                if (!out.entries.empty()) pl.rounds.push_back(std::move(out));
            }
            if (c.s > 0) pl.rounds.push_back(std::move(deliver));
            break;
        }
        case ISO_ALG_ONEHOP: {
            if (c.mesh) return ISO_ERR_ARG;
            // one launch per unit of coordinate: refuse neighbourhoods whose raw coordinates
            // would need an absurd number of them (and keep the hop arithmetic inside int32)
            int64_t steps = 0;
            for (int j = 0; j < c.d; ++j) {
                int64_t up = 0, down = 0;
                for (int i = 0; i < c.s; ++i) {
                    const int64_t v = c.raw[(size_t)i * c.d + j];
                    up = std::max(up, v);
                    down = std::max(down, -v);
                }
                steps += up + down;
            }
            if (steps > kMaxOneHopRounds) return ISO_ERR_TOO_LARGE;
            if (op == ISO_OP_ALLTOALL)
                plan_alltoall_onehop(c, pl);
            else
                plan_allgather_onehop(c, pl);
            break;
        }
        case ISO_ALG_SX_ROUNDS:
        case ISO_ALG_SX_FUSED:
            plan_s_exchange(c, op, algorithm == ISO_ALG_SX_FUSED, pl);
            break;
        default:
            return ISO_ERR_ARG;
    }
    for (Round &r : pl.rounds)
        if (r.kind != ISO_ROUND_DELIVER)
            for (iso_plan_entry_t &e : r.entries) e.dim = r.kind == ISO_ROUND_SHIFT ? r.dim : -1;
    out = std::move(pl);
    return ISO_SUCCESS;
}

}  // namespace iso
