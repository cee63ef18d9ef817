"""CPU oracle for isomorphic sparse all-to-all and allgather on a torus.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module;
only tests/, the smoke check and the benchmark's cpu_baseline leg do.  It shares
no code with the HIP library: the only common code is the seeded input
generators in `iso_inputs`, which contain none of the method's arithmetic.

Part 1 is the plain definition of what the collectives compute (Section 2 of
the paper): process R sends its i-th block to R (+) C^i, hence receives its i-th
block from R (-) C^i, with component-wise wrap-around.  The message-combining
schedules reach exactly this result, so the definition is the oracle.

Part 2 counts rounds and block-moves of the schedules (Sections 3.1, 3.2, 5).

Part 3 replays the message-combining schedules themselves, process by process,
with explicit send / receive / intermediate buffers, taking the steps in the
paper's order (Algorithm 1's alternating-buffer rule; Section 3.2's prefix
trie; Section 5's one-round-per-distinct-coordinate variant).  Tests use it to
show that the combined schedules give the same result as the definition.

Readings of points the paper leaves open:
  * rank <-> coordinate: row-major, last dimension fastest (the MPI Cartesian
    convention the paper's library sits on).
  * coordinates are reduced modulo the dimension size before any counting; a
    coordinate congruent to zero needs no hop.
  * the zero vector and repeated vectors are legal (Section 2); a zero vector
    is a same-process copy.
  * allgather volume W counts each trie edge once (so that W <= V holds).

Every function is pinned by tests/test_oracle.py against something other than
itself (numpy.roll, brute-force push simulation, closed forms and the numbers
the paper prints); nothing here is "parity unpinned".
"""
import numpy as np


# ---------------------------------------------------------------------------
# Part 1: the definition (Section 2)
# ---------------------------------------------------------------------------

def rank_to_coords(ranks, dims):
    """Row-major unflatten, last dimension fastest: int64 array (..., d)."""
    ranks = np.asarray(ranks, dtype=np.int64)
    out = np.empty(ranks.shape + (len(dims),), dtype=np.int64)
    rem = ranks.copy()
    for j in range(len(dims) - 1, -1, -1):
        out[..., j] = rem % dims[j]
        rem //= dims[j]
    return out


def coords_to_rank(coords, dims):
    coords = np.asarray(coords, dtype=np.int64)
    r = np.zeros(coords.shape[:-1], dtype=np.int64)
    for j in range(len(dims)):
        r = r * dims[j] + coords[..., j]
    return r


def torus_add(R, C, dims):
    """R (+) C: component-wise sum modulo the dimension sizes (Section 2)."""
    return np.mod(np.asarray(R, dtype=np.int64) + np.asarray(C, dtype=np.int64),
                  np.asarray(dims, dtype=np.int64))


def torus_sub(R, C, dims):
    """R (-) C, result in [0, p_j) in every component."""
    return np.mod(np.asarray(R, dtype=np.int64) - np.asarray(C, dtype=np.int64),
                  np.asarray(dims, dtype=np.int64))


def source_ranks(dims, offsets, ranks=None):
    """int64 (len(ranks), s): rank of R (-) C^i, the process whose i-th block
    process R receives (Section 2)."""
    p = int(np.prod(dims, dtype=np.int64))
    ranks = np.arange(p, dtype=np.int64) if ranks is None else np.asarray(ranks, np.int64)
    offs = np.asarray(offsets, dtype=np.int64).reshape(-1, len(dims))
    rc = rank_to_coords(ranks, dims)                       # (n, d)
    src = torus_sub(rc[:, None, :], offs[None, :, :], dims)  # (n, s, d)
    return coords_to_rank(src, dims)


def target_ranks(dims, offsets, ranks=None):
    """int64 (len(ranks), s): rank of R (+) C^i (Section 2)."""
    p = int(np.prod(dims, dtype=np.int64))
    ranks = np.arange(p, dtype=np.int64) if ranks is None else np.asarray(ranks, np.int64)
    offs = np.asarray(offsets, dtype=np.int64).reshape(-1, len(dims))
    rc = rank_to_coords(ranks, dims)
    return coords_to_rank(torus_add(rc[:, None, :], offs[None, :, :], dims), dims)


def alltoall(dims, offsets, send):
    """recv[R][i] = send[R (-) C^i][i].  send: array (p, s, ...) -> same shape.
    Blocks sit in neighbour order in both buffers (Section 2)."""
    send = np.asarray(send)
    s = len(offsets)
    src = source_ranks(dims, offsets)
    assert send.shape[0] == src.shape[0] and send.shape[1] == s
    recv = np.empty_like(send)
    for i in range(s):
        recv[:, i] = send[src[:, i], i]
    return recv


def allgather(dims, offsets, send):
    """recv[R][i] = send[R (-) C^i].  send: (p, ...) -> recv (p, s, ...)."""
    send = np.asarray(send)
    s = len(offsets)
    src = source_ranks(dims, offsets)
    assert send.shape[0] == src.shape[0]
    recv = np.empty((send.shape[0], s) + send.shape[1:], dtype=send.dtype)
    for i in range(s):
        recv[:, i] = send[src[:, i]]
    return recv


# ---------------------------------------------------------------------------
# Part 2: schedule metrics
# ---------------------------------------------------------------------------

def canonical(dims, offsets):
    """Offsets reduced into [0, p_j): list of tuples."""
    return [tuple(int(c) % int(pj) for c, pj in zip(C, dims)) for C in offsets]


def direct_rounds(dims, offsets):
    """List of (j, v) rounds of the torus-direct schedules (Section 5): for each
    dimension, one round per distinct non-zero coordinate value."""
    can = canonical(dims, offsets)
    rounds = []
    for j in range(len(dims)):
        for v in sorted({C[j] for C in can} - {0}):
            rounds.append((j, v))
    return rounds


def direct_alltoall_volume(dims, offsets):
    """Blocks sent per process by torus-direct all-to-all: each block makes one
    hop per non-zero coordinate (Section 5)."""
    return sum(sum(1 for c in C if c) for C in canonical(dims, offsets))


def trie_edges(dims, offsets, order=None):
    """Non-zero edges of the prefix trie over the (reduced) offsets taken in
    dimension order `order` (Section 3.2): set of prefixes (tuples of length
    t+1 over the first t+1 dimensions of the order) whose last entry is
    non-zero.  Each such prefix is one block that a process receives once."""
    d = len(dims)
    order = list(range(d)) if order is None else list(order)
    can = canonical(dims, offsets)
    return {tuple(C[order[u]] for u in range(t + 1))
            for C in can for t in range(d) if C[order[t]] != 0}


def direct_allgather_volume(dims, offsets, order=None):
    """Distinct blocks received per process by torus-direct allgather = number of
    non-zero trie edges.  (Repeated offsets share their trie path.)"""
    return len(trie_edges(dims, offsets, order))


def onehop_rounds(offsets):
    """D of Proposition 1: sum over dimensions of the largest positive plus the
    largest negative excursion (raw, unreduced coordinates)."""
    offs = np.asarray(offsets, dtype=np.int64)
    if offs.size == 0:
        return 0
    return int(np.maximum(offs, 0).max(axis=0).sum() + np.maximum(-offs, 0).max(axis=0).sum())


def onehop_alltoall_volume(offsets):
    """V = sum of the 1-norms (Section 3.1)."""
    return int(np.abs(np.asarray(offsets, dtype=np.int64)).sum())


def onehop_allgather_volume(offsets, order=None):
    """W for the one-hop torus allgather: total |weight| over distinct trie edges
    (Section 3.2; edges counted once each so that W <= V)."""
    offs = [tuple(int(c) for c in C) for C in offsets]
    if not offs:
        return 0
    d = len(offs[0])
    order = list(range(d)) if order is None else list(order)
    edges = {tuple(C[order[u]] for u in range(t + 1)) for C in offs for t in range(d)}
    return sum(abs(e[-1]) for e in edges)


# ---------------------------------------------------------------------------
# Part 3: replay of the message-combining schedules, process by process
# ---------------------------------------------------------------------------

def _shift_push(buf_rows, dims, j, v):
    """Every process R hands `buf_rows[R]` to process R (+) v*e_j; returns the
    array indexed by the receiving process."""
    p = buf_rows.shape[0]
    e = np.zeros(len(dims), dtype=np.int64)
    e[j] = v
    tgt = coords_to_rank(torus_add(rank_to_coords(np.arange(p), dims), e, dims), dims)
    out = np.empty_like(buf_rows)
    out[tgt] = buf_rows
    return out


def replay_direct_alltoall(dims, offsets, send, return_trace=False):
    """Torus-direct all-to-all with Algorithm 1's alternating buffers.

    hops[i] starts as the number of non-zero coordinates of C^i (Section 5).
    In the round for (dimension j, value v) every block i with c^i_j == v is
    sent from where it currently sits (the send buffer if j is the block's first
    non-zero dimension) to process R (+) v*e_j, which receives it into the
    intermediate buffer if hops[i] is even and into the receive buffer if odd;
    then hops[i] drops by one.  Zero vectors are same-process copies."""
    send = np.asarray(send)
    p, s = send.shape[0], len(offsets)
    can = canonical(dims, offsets)
    recvbuf = np.zeros_like(send)
    interbuf = np.zeros_like(send)
    where = ["send"] * s
    hops = [sum(1 for c in C if c) for C in can]
    trace = []
    bufs = {"send": send, "recv": recvbuf, "inter": interbuf}
    for i in range(s):
        if hops[i] == 0:
            recvbuf[:, i] = send[:, i]
            where[i] = "recv"
    for (j, v) in direct_rounds(dims, offsets):
        parts = []
        for i in range(s):
            if can[i][j] != v:
                continue
            dst = "inter" if hops[i] % 2 == 0 else "recv"
            parts.append((i, where[i], dst))
        # all sends of the round read the old buffers, then all receives land
        landed = [(i, dst, _shift_push(bufs[src][:, i], dims, j, v)) for i, src, dst in parts]
        for i, dst, data in landed:
            bufs[dst][:, i] = data
            where[i] = dst
            hops[i] -= 1
        trace.append(((j, v), parts))
    assert all(h == 0 for h in hops) and all(w == "recv" for w in where)
    return (recvbuf, trace) if return_trace else recvbuf


def replay_direct_allgather(dims, offsets, send, order=None):
    """Torus-direct allgather along the prefix trie (Sections 3.2 and 5).

    A trie node with prefix P (over the first t+1 dimensions of `order`) stands
    for the block that came from process R (-) P.  It is obtained, in the round
    of dimension order[t] and value P[t], from the node for prefix P[:t] held
    by the process P[t] steps back in that dimension; a zero edge keeps the
    block where it is.  Leaves are the s received blocks."""
    send = np.asarray(send)
    p, s, d = send.shape[0], len(offsets), len(dims)
    order = list(range(d)) if order is None else list(order)
    can = canonical(dims, offsets)
    node = {(): send}                       # prefix -> array indexed by process
    for t in range(d):
        j = order[t]
        prefixes = sorted({tuple(C[order[u]] for u in range(t + 1)) for C in can})
        new = {}
        for v in sorted({P[-1] for P in prefixes}):
            for P in prefixes:
                if P[-1] != v:
                    continue
                parent = node[P[:-1]]
                new[P] = parent if v == 0 else _shift_push(parent, dims, j, v)
        node = new
    recv = np.empty((p, s) + send.shape[1:], dtype=send.dtype)
    for i, C in enumerate(can):
        recv[:, i] = node[tuple(C[order[u]] for u in range(d))]
    return recv


def replay_s_exchange_alltoall(dims, offsets, send):
    """The straightforward s-round algorithm (Section 3, first listing): in
    round i every process sends block i to R (+) C^i and receives block i from
    R (-) C^i."""
    send = np.asarray(send)
    tgt = target_ranks(dims, offsets)
    recv = np.empty_like(send)
    for i in range(len(offsets)):
        recv[tgt[:, i], i] = send[:, i]
    return recv


def onehop_steps(offsets):
    """The D communication steps of the one-ported torus schedules (Section 3.1,
    Algorithm 1): per dimension j, first max_i c^i_j steps in the positive
    direction, then max_i (-c^i_j) steps in the negative one.  List of
    (j, direction, h)."""
    offs = np.asarray(offsets, dtype=np.int64)
    steps = []
    if offs.size == 0:
        return steps
    for j in range(offs.shape[1]):
        for h in range(int(max(0, offs[:, j].max()))):
            steps.append((j, +1, h))
        for h in range(int(max(0, (-offs[:, j]).max()))):
            steps.append((j, -1, h))
    return steps


def replay_onehop_alltoall(dims, offsets, send, return_trace=False):
    """One-ported torus all-to-all with alternating buffers (Algorithm 1).

    hops[i] = ||C^i|| (raw coordinates).  In step h of dimension j, direction
    +1, every block with c^i_j > h moves one hop to R (+) e_j (direction -1:
    blocks with -c^i_j > h move to R (-) e_j).  It is received into the
    intermediate buffer if hops[i] is even, into the receive buffer if odd, and
    is sent from the send buffer on its very first hop, afterwards from the
    buffer it was last received into.  (The printed algorithm names the send
    buffer for every step of a block's first dimension; only the first hop can
    be meant, since later steps must forward what the previous step delivered.)"""
    send = np.asarray(send)
    s = len(offsets)
    offs = [tuple(int(c) for c in C) for C in offsets]
    recvbuf, interbuf = np.zeros_like(send), np.zeros_like(send)
    bufs = {"send": send, "recv": recvbuf, "inter": interbuf}
    where = ["send"] * s
    hops = [sum(abs(c) for c in C) for C in offs]
    for i in range(s):
        if hops[i] == 0:
            recvbuf[:, i] = send[:, i]
            where[i] = "recv"
    trace = []
    for (j, sign, h) in onehop_steps(offs):
        parts = []
        for i in range(s):
            if sign * offs[i][j] > h:
                parts.append((i, where[i], "inter" if hops[i] % 2 == 0 else "recv"))
        landed = [(i, dst, _shift_push(bufs[src][:, i], dims, j, sign)) for i, src, dst in parts]
        for i, dst, data in landed:
            bufs[dst][:, i] = data
            where[i] = dst
            hops[i] -= 1
        trace.append(((j, sign, h), parts))
    assert all(x == 0 for x in hops) and all(w == "recv" for w in where)
    return (recvbuf, trace) if return_trace else recvbuf


def replay_onehop_allgather(dims, offsets, send, order=None, return_moves=False):
    """One-ported torus allgather along the prefix trie (Section 3.2): in step h
    of dimension order[t], direction +1, every trie node at level t whose edge
    weight c exceeds h advances one hop (direction -1: -c > h).  Nodes start as
    a copy of their parent's block; zero edges do not move."""
    send = np.asarray(send)
    p, s = send.shape[0], len(offsets)
    offs = [tuple(int(c) for c in C) for C in offsets]
    d = len(dims)
    order = list(range(d)) if order is None else list(order)
    node = {(): send}
    moves = 0
    for t in range(d):
        j = order[t]
        prefixes = sorted({tuple(C[order[u]] for u in range(t + 1)) for C in offs})
        cur = {P: node[P[:-1]] for P in prefixes}
        pos = max([P[-1] for P in prefixes] + [0])
        neg = max([-P[-1] for P in prefixes] + [0])
        for sign, count in ((+1, pos), (-1, neg)):
            for h in range(count):
                for P in prefixes:
                    if sign * P[-1] > h:
                        cur[P] = _shift_push(cur[P], dims, j, sign)
                        moves += 1
        node = cur
    recv = np.empty((p, s) + send.shape[1:], dtype=send.dtype)
    for i, C in enumerate(offs):
        recv[:, i] = node[tuple(C[order[u]] for u in range(d))]
    return (recv, moves) if return_moves else recv


# ---------------------------------------------------------------------------
# Part 4: irregular variants (Section 2, second interface listing): per-neighbour
# block sizes and displacements, identical on all processes, send and receive
# sizes equal pairwise
# ---------------------------------------------------------------------------

def alltoallv(dims, offsets, send_rows, sizes, send_displs, recv_rows, recv_displs):
    """recv_rows[R][recv_displs[i] : +sizes[i]] = send_rows[R (-) C^i][send_displs[i] : +sizes[i]].
    send_rows: uint8 (p, send_extent); recv_rows: uint8 (p, recv_extent), modified in
    place and returned (bytes outside the s blocks keep their value)."""
    src = source_ranks(dims, offsets)
    for i in range(len(offsets)):
        n = int(sizes[i])
        recv_rows[:, recv_displs[i]:recv_displs[i] + n] = \
            send_rows[src[:, i], send_displs[i]:send_displs[i] + n]
    return recv_rows


def allgatherv(dims, offsets, send_rows, size, recv_rows, recv_displs):
    """recv_rows[R][recv_displs[i] : +size] = send_rows[R (-) C^i][0 : size]."""
    src = source_ranks(dims, offsets)
    for i in range(len(offsets)):
        recv_rows[:, recv_displs[i]:recv_displs[i] + size] = send_rows[src[:, i], :size]
    return recv_rows


# ---------------------------------------------------------------------------
# Part 5: meshes (Section 7: dimensions may be non-periodic, as in an MPI
# Cartesian topology).  In a non-periodic dimension nothing wraps: a process
# whose source R - C^i would lie outside the mesh receives nothing for
# neighbour i and its i-th receive block keeps its content.
# ---------------------------------------------------------------------------

def source_ranks_mesh(dims, periodic, offsets, ranks=None):
    """(src, valid): int64 (n, s) source ranks and bool (n, s) "a source exists".
    Periodic dimensions wrap as on the torus; in the others R - C^i must stay in
    [0, p_j), using the coordinate as given (no reduction)."""
    dims_a = np.asarray(dims, dtype=np.int64)
    per = np.asarray(periodic, dtype=bool)
    p = int(np.prod(dims_a))
    ranks = np.arange(p, dtype=np.int64) if ranks is None else np.asarray(ranks, np.int64)
    offs = np.asarray(offsets, dtype=np.int64).reshape(-1, len(dims))
    raw = rank_to_coords(ranks, dims)[:, None, :] - offs[None, :, :]          # (n, s, d)
    inside = (raw >= 0) & (raw < dims_a)
    valid = np.all(inside | per, axis=2)
    src = coords_to_rank(np.where(per, np.mod(raw, dims_a), np.clip(raw, 0, dims_a - 1)), dims)
    return src, valid


def alltoall_mesh(dims, periodic, offsets, send, recv):
    """recv[R][i] = send[R - C^i][i] where that source exists; other blocks of
    `recv` (modified in place, returned) keep their content."""
    src, valid = source_ranks_mesh(dims, periodic, offsets)
    for i in range(len(offsets)):
        v = valid[:, i]
        recv[v, i] = send[src[v, i], i]
    return recv


def allgather_mesh(dims, periodic, offsets, send, recv):
    src, valid = source_ranks_mesh(dims, periodic, offsets)
    for i in range(len(offsets)):
        v = valid[:, i]
        recv[v, i] = send[src[v, i]]
    return recv
