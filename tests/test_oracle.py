"""Pins for the CPU oracle: every function of oracle/iso_oracle.py is checked
against something other than itself -- numpy.roll (a library routine that is
the definition's special case per slot), a pure-Python push simulation of the
p processes, closed forms, and the values the paper prints."""
import itertools

import numpy as np
import pytest

import iso_inputs as gen
from oracle import iso_oracle as orc
from oracle import c_twin

RNG = np.random.default_rng(20160624)

TORI = [
    ((5,), [(1,), (-2,), (7,)]),
    ((4, 3), [(1, 0), (0, -1), (1, 1), (-1, 2), (0, 0), (1, 1)]),
    ((3, 2, 4), gen.moore(3, 1)),
    ((2, 1, 5), [(1, 0, 2), (0, 3, -1), (-5, 0, 6), (0, 0, 0)]),
    ((2, 2, 2, 2), gen.moore(4, 1)),            # s = 80 > p = 16: heavy aliasing
    ((6, 5), gen.von_neumann(2, 2)),
    ((7, 3, 2), gen.positive_octant(3, 3)),
]


def _rand_send(p, s, m):
    return RNG.integers(0, 256, size=(p, s, m), dtype=np.uint8)


# ---------------------------------------------------------------- definition

@pytest.mark.parametrize("dims,offsets", TORI)
def test_alltoall_equals_numpy_roll_per_slot(dims, offsets):
    p, s = int(np.prod(dims)), len(offsets)
    send = _rand_send(p, s, 6)
    recv = orc.alltoall(dims, offsets, send)
    axes = tuple(range(len(dims)))
    for i, C in enumerate(offsets):
        grid = send[:, i].reshape(tuple(dims) + (6,))
        want = np.roll(grid, shift=tuple(C), axis=axes).reshape(p, 6)
        assert np.array_equal(recv[:, i], want), f"slot {i} offset {C}"


@pytest.mark.parametrize("dims,offsets", TORI)
def test_allgather_equals_numpy_roll(dims, offsets):
    p = int(np.prod(dims))
    send = RNG.integers(0, 256, size=(p, 5), dtype=np.uint8)
    recv = orc.allgather(dims, offsets, send)
    axes = tuple(range(len(dims)))
    for i, C in enumerate(offsets):
        want = np.roll(send.reshape(tuple(dims) + (5,)), shift=tuple(C), axis=axes).reshape(p, 5)
        assert np.array_equal(recv[:, i], want)


def _push_brute_force(dims, offsets, send, allgather=False):
    """p processes, each pushing its blocks to R (+) C^i, in pure Python."""
    d = len(dims)
    coords = list(itertools.product(*[range(n) for n in dims]))   # row-major order
    index = {c: r for r, c in enumerate(coords)}
    recv = [[None] * len(offsets) for _ in coords]
    for R, rc in enumerate(coords):
        for i, C in enumerate(offsets):
            tgt = tuple((rc[j] + C[j]) % dims[j] for j in range(d))
            recv[index[tgt]][i] = send[R] if allgather else send[R][i]
    return recv


@pytest.mark.parametrize("dims,offsets", [t for t in TORI if np.prod(t[0]) <= 48])
def test_pull_definition_equals_push_brute_force(dims, offsets):
    p, s = int(np.prod(dims)), len(offsets)
    send = _rand_send(p, s, 3)
    want = _push_brute_force(dims, offsets, send)
    got = orc.alltoall(dims, offsets, send)
    for R in range(p):
        for i in range(s):
            assert np.array_equal(got[R, i], want[R][i]), (R, i)
    sg = send[:, 0]
    wantg = _push_brute_force(dims, offsets, sg, allgather=True)
    gotg = orc.allgather(dims, offsets, sg)
    for R in range(p):
        for i in range(s):
            assert np.array_equal(gotg[R, i], wantg[R][i]), (R, i)


def test_rank_linearisation_is_row_major_last_fastest():
    dims = (3, 4, 5)
    want = np.array(list(itertools.product(range(3), range(4), range(5))))
    assert np.array_equal(orc.rank_to_coords(np.arange(60), dims), want)
    assert np.array_equal(orc.coords_to_rank(want, dims), np.arange(60))
    # explicit spot values: rank = (r0*4 + r1)*5 + r2
    assert orc.coords_to_rank(np.array([2, 1, 3]), dims) == 48


def test_source_of_a_single_known_case():
    # 1-d ring of 5, offset +2: process 0 receives from process 3 (= 0 - 2 mod 5)
    assert orc.source_ranks((5,), [(2,)])[0, 0] == 3
    assert orc.target_ranks((5,), [(2,)])[0, 0] == 2
    # 2-d 3x4, offset (1,-1): process (0,0) receives from (2,1) = rank 9
    assert orc.source_ranks((3, 4), [(1, -1)])[0, 0] == 9


@pytest.mark.parametrize("dims,offsets", TORI)
def test_inverse_neighbourhood_returns_send(dims, offsets):
    p, s = int(np.prod(dims)), len(offsets)
    send = _rand_send(p, s, 4)
    neg = [tuple(-c for c in C) for C in offsets]
    back = orc.alltoall(dims, neg, orc.alltoall(dims, offsets, send))
    assert np.array_equal(back, send)


@pytest.mark.parametrize("dims,offsets", TORI)
def test_allgather_is_alltoall_of_replicated_block(dims, offsets):
    p, s = int(np.prod(dims)), len(offsets)
    one = RNG.integers(0, 256, size=(p, 4), dtype=np.uint8)
    rep = np.repeat(one[:, None, :], s, axis=1)
    assert np.array_equal(orc.allgather(dims, offsets, one), orc.alltoall(dims, offsets, rep))


def test_translation_equivariance():
    dims, offsets = (4, 3, 5), gen.moore(3, 1)
    p, s = 60, 26
    send = _rand_send(p, s, 2)
    T = (1, 2, 3)
    axes = (0, 1, 2)

    def roll_ranks(a):
        return np.roll(a.reshape(dims + a.shape[1:]), T, axis=axes).reshape(a.shape)

    assert np.array_equal(orc.alltoall(dims, offsets, roll_ranks(send)),
                          roll_ranks(orc.alltoall(dims, offsets, send)))


def test_planted_mistakes_are_caught_by_the_pins():
    """The pins have teeth: swapping (-) for (+), or transposing the rank
    linearisation, makes the numpy.roll comparison fail."""
    dims, offsets = (4, 3), [(1, 0), (0, 1), (1, 2)]
    p, s = 12, 3
    send = _rand_send(p, s, 4)
    good = orc.alltoall(dims, offsets, send)

    wrong_sign = np.empty_like(send)
    tgt = orc.target_ranks(dims, offsets)
    for i in range(s):
        wrong_sign[:, i] = send[tgt[:, i], i]
    assert not np.array_equal(wrong_sign, good)

    col_major = np.empty_like(send)       # first dimension fastest
    for R in range(p):
        rc = (R % 4, R // 4)
        for i, C in enumerate(offsets):
            sc = ((rc[0] - C[0]) % 4, (rc[1] - C[1]) % 3)
            col_major[R, i] = send[sc[0] + 4 * sc[1], i]
    assert not np.array_equal(col_major, good)

    for i, C in enumerate(offsets):
        want = np.roll(send[:, i].reshape(4, 3, 4), C, axis=(0, 1)).reshape(p, 4)
        assert np.array_equal(good[:, i], want)
        assert not np.array_equal(wrong_sign[:, i], want)
        assert not np.array_equal(col_major[:, i], want)


# ---------------------------------------------------------------- metrics

def _ints(text, sep=","):
    return [int(x) for x in text.split(sep) if x.strip()]


def test_generators_match_printed_neighbour_counts(golden):
    for item in golden["moore_counts"].split(","):
        d, r, n = (int(x) for x in item.strip().split(":"))
        assert len(gen.moore(d, r)) == n == (2 * r + 1) ** d - 1
    assert len(gen.positive_octant(3, 3)) == int(golden["positive_octant_d3_r3"])
    assert len(gen.shales(3, (3, 7))) == int(golden["shales_d3_r3_r7"])
    flat = _ints(golden["octant_flat"])
    s, d = int(golden["octant_s"]), int(golden["octant_d"])
    assert len(flat) == s * d
    octant = {tuple(flat[i * d:(i + 1) * d]) for i in range(s)}
    assert octant == set(gen.positive_octant(3, 1))


def test_round_counts_printed_in_the_paper(golden):
    big = (64,) * 5
    m3 = gen.moore(3, 1)
    assert len(m3) == int(golden["stencil27_neighbours"])
    assert len(orc.direct_rounds(big[:3], m3)) == int(golden["stencil27_rounds"])
    assert orc.onehop_rounds(m3) == int(golden["stencil27_rounds"])
    for d in (2, 3, 4):
        for r in (1, 2, 3):
            offs = gen.moore(d, r)
            assert orc.onehop_rounds(offs) == 2 * r * d
            assert len(orc.direct_rounds(big[:d], offs)) == 2 * r * d
    flat = _ints(golden["octant_flat"])
    octant = [tuple(flat[i * 3:(i + 1) * 3]) for i in range(7)]
    assert len(orc.direct_rounds((8, 8, 8), octant)) == 3


def test_moore_volume_closed_forms():
    for d, r in [(2, 1), (3, 1), (3, 2), (4, 1), (2, 3)]:
        offs = gen.moore(d, r)
        dims = (4 * r + 3,) * d
        s = len(offs)
        assert orc.direct_alltoall_volume(dims, offs) == 2 * r * d * (2 * r + 1) ** (d - 1)
        assert orc.direct_allgather_volume(dims, offs) == s
        # one-hop all-to-all volume: sum of 1-norms = d (2r+1)^(d-1) r (r+1)
        assert orc.onehop_alltoall_volume(offs) == d * (2 * r + 1) ** (d - 1) * r * (r + 1)
    assert orc.direct_alltoall_volume((32, 32, 32), gen.moore(3, 1)) == 54
    assert orc.direct_alltoall_volume((256, 256), gen.von_neumann(2, 2)) == 16


def test_figure1_trie_example(golden):
    offs = [tuple(_ints(t)) for t in golden["fig1_offsets"].split(";")]
    dims = (16, 16, 16)
    assert orc.onehop_rounds(offs) == int(golden["fig1_onehop_D"])
    assert orc.onehop_alltoall_volume(offs) == int(golden["fig1_onehop_V"])
    assert orc.onehop_allgather_volume(offs) == int(golden["fig1_onehop_W"])
    rounds = orc.direct_rounds(dims, offs)
    assert len(rounds) == int(golden["fig1_direct_rounds"])
    assert orc.direct_alltoall_volume(dims, offs) == int(golden["fig1_direct_V"])
    assert orc.direct_allgather_volume(dims, offs) == int(golden["fig1_direct_W"])
    edges = orc.trie_edges(dims, offs)
    k_ag = [sum(1 for e in edges if len(e) == j + 1 and e[-1] == v) for j, v in rounds]
    assert k_ag == _ints(golden["fig1_direct_allgather_k"])
    _, trace = orc.replay_direct_alltoall(dims, offs, np.zeros((16 ** 3, 10, 1), np.uint8),
                                          return_trace=True)
    assert [len(parts) for _, parts in trace] == _ints(golden["fig1_direct_alltoall_k"])


@pytest.mark.parametrize("dims,offsets", TORI)
def test_volume_invariants(dims, offsets):
    V = orc.direct_alltoall_volume(dims, offsets)
    W = orc.direct_allgather_volume(dims, offsets)
    assert W <= V
    assert orc.onehop_allgather_volume(offsets) <= orc.onehop_alltoall_volume(offsets)
    rounds = orc.direct_rounds(dims, offsets)
    assert len(rounds) <= sum(min(len(offsets), n - 1) for n in dims)
    # coordinates congruent modulo the dimension size count once
    shifted = [tuple(c + n for c, n in zip(C, dims)) for C in offsets]
    assert orc.direct_rounds(dims, shifted) == rounds


# ---------------------------------------------------------------- schedule replays

@pytest.mark.parametrize("dims,offsets", TORI)
def test_combined_alltoall_schedule_reaches_the_definition(dims, offsets):
    p, s = int(np.prod(dims)), len(offsets)
    send = _rand_send(p, s, 3)
    keep = send.copy()
    recv, trace = orc.replay_direct_alltoall(dims, offsets, send, return_trace=True)
    assert np.array_equal(recv, orc.alltoall(dims, offsets, send))
    assert np.array_equal(send, keep)                       # send buffer untouched
    assert len(trace) == len(orc.direct_rounds(dims, offsets))
    can = orc.canonical(dims, offsets)
    seen_inter = set()
    for (j, v), parts in trace:
        for i, src, dst in parts:
            assert src != dst
            if dst == "inter":
                seen_inter.add(i)
    for i, C in enumerate(can):
        nnz = sum(1 for c in C if c)
        assert (i in seen_inter) == (nnz >= 2)              # single hops go send -> recv


@pytest.mark.parametrize("dims,offsets", TORI)
def test_combined_allgather_schedule_reaches_the_definition(dims, offsets):
    p = int(np.prod(dims))
    send = RNG.integers(0, 256, size=(p, 3), dtype=np.uint8)
    want = orc.allgather(dims, offsets, send)
    assert np.array_equal(orc.replay_direct_allgather(dims, offsets, send), want)
    order = list(range(len(dims)))[::-1]
    assert np.array_equal(orc.replay_direct_allgather(dims, offsets, send, order), want)


@pytest.mark.parametrize("dims,offsets", TORI)
def test_s_exchange_equals_definition(dims, offsets):
    p, s = int(np.prod(dims)), len(offsets)
    send = _rand_send(p, s, 3)
    assert np.array_equal(orc.replay_s_exchange_alltoall(dims, offsets, send),
                          orc.alltoall(dims, offsets, send))


def test_combined_equals_direct_on_config_1_and_2_inputs():
    for key, m in ((1, None), (2, 16)):          # config 2 with short blocks: same routing
        cfg = gen.get_config(key)
        m = m or cfg.m
        send = gen.alltoall_send(11, cfg.p, cfg.s, m, cfg.kind)
        want = orc.alltoall(cfg.dims, cfg.offsets, send)
        assert np.array_equal(orc.replay_direct_alltoall(cfg.dims, cfg.offsets, send), want)
        one = gen.allgather_send(11, cfg.p, m, cfg.kind)
        assert np.array_equal(orc.replay_direct_allgather(cfg.dims, cfg.offsets, one),
                              orc.allgather(cfg.dims, cfg.offsets, one))


# ---------------------------------------------------------------- C twin

@pytest.mark.parametrize("dims,offsets", TORI)
def test_c_twin_matches_numpy_oracle(dims, offsets):
    p, s = int(np.prod(dims)), len(offsets)
    for m in (1, 7, 16, 40):
        send = _rand_send(p, s, m)
        got, used = c_twin.alltoall(dims, offsets, send, threads=2)
        assert used >= 1
        assert np.array_equal(got, orc.alltoall(dims, offsets, send))
        one = np.ascontiguousarray(send[:, 0])
        gotg, _ = c_twin.allgather(dims, offsets, one, threads=1)
        assert np.array_equal(gotg, orc.allgather(dims, offsets, one))


def test_c_twin_config1_against_roll():
    cfg = gen.get_config(1)
    send = gen.alltoall_send(5, cfg.p, cfg.s, cfg.m)
    got, _ = c_twin.alltoall(cfg.dims, cfg.offsets, send)
    for i, C in enumerate(cfg.offsets):
        want = np.roll(send[:, i].reshape(cfg.dims + (cfg.m,)), C, axis=(0, 1)).reshape(cfg.p, cfg.m)
        assert np.array_equal(got[:, i], want)


# ---------------------------------------------------------------- one-hop torus schedules

@pytest.mark.parametrize("dims,offsets", TORI)
def test_onehop_schedules_reach_the_definition(dims, offsets):
    p, s = int(np.prod(dims)), len(offsets)
    send = _rand_send(p, s, 3)
    keep = send.copy()
    recv, trace = orc.replay_onehop_alltoall(dims, offsets, send, return_trace=True)
    assert np.array_equal(recv, orc.alltoall(dims, offsets, send))
    assert np.array_equal(send, keep)
    # Proposition 1: D steps, V block-moves, every step moves at least one block
    assert len(trace) == orc.onehop_rounds(offsets) == len(orc.onehop_steps(offsets))
    assert sum(len(parts) for _, parts in trace) == orc.onehop_alltoall_volume(offsets)
    assert all(parts for _, parts in trace)
    one = np.ascontiguousarray(send[:, 0])
    got, moves = orc.replay_onehop_allgather(dims, offsets, one, return_moves=True)
    assert np.array_equal(got, orc.allgather(dims, offsets, one))
    # Proposition 2: W block-moves, W <= V
    assert moves == orc.onehop_allgather_volume(offsets) <= orc.onehop_alltoall_volume(offsets)


def test_onehop_figure1_counts(golden):
    offs = [tuple(_ints(t)) for t in golden["fig1_offsets"].split(";")]
    dims = (6, 5, 4)
    send = _rand_send(120, 10, 2)
    _, trace = orc.replay_onehop_alltoall(dims, offs, send, return_trace=True)
    assert len(trace) == int(golden["fig1_onehop_D"])
    assert sum(len(p) for _, p in trace) == int(golden["fig1_onehop_V"])
    _, moves = orc.replay_onehop_allgather(dims, offs, send[:, 0], return_moves=True)
    assert moves == int(golden["fig1_onehop_W"])


# ---------------------------------------------------------------- irregular variants

def test_irregular_reduces_to_regular_and_to_roll(golden):
    dims, offsets = (4, 3, 5), gen.moore(3, 1)
    p, s, m = 60, 26, 8
    send = _rand_send(p, s, m)
    displs = [i * m for i in range(s)]
    recv = np.zeros((p, s * m), np.uint8)
    orc.alltoallv(dims, offsets, send.reshape(p, s * m), [m] * s, displs, recv, displs)
    assert np.array_equal(recv.reshape(p, s, m), orc.alltoall(dims, offsets, send))
    # genuinely irregular: stencil sizes, padded displacements on the send side, reversed order on the
    # receive side; every block checked against numpy.roll, every other byte must keep its value
    sizes = gen.stencil_block_sizes(offsets, 3)
    sd, sext = gen.packed_displacements(sizes, 4)
    order = list(range(s))[::-1]
    rd, at = [0] * s, 5
    for i in order:
        rd[i] = at
        at += sizes[i] + 2
    rext = at + 3
    send_rows = RNG.integers(0, 256, size=(p, sext), dtype=np.uint8)
    recv_rows = np.full((p, rext), 0xEE, np.uint8)
    orc.alltoallv(dims, offsets, send_rows, sizes, sd, recv_rows, rd)
    covered = np.zeros(rext, bool)
    for i, C in enumerate(offsets):
        blk = send_rows[:, sd[i]:sd[i] + sizes[i]].reshape(dims + (sizes[i],))
        want = np.roll(blk, C, axis=(0, 1, 2)).reshape(p, sizes[i])
        assert np.array_equal(recv_rows[:, rd[i]:rd[i] + sizes[i]], want)
        covered[rd[i]:rd[i] + sizes[i]] = True
    assert (recv_rows[:, ~covered] == 0xEE).all()
    # allgather with displacements
    one = RNG.integers(0, 256, size=(p, 7), dtype=np.uint8)
    rows = np.full((p, rext), 0xEE, np.uint8)
    gd = [3 + 9 * i for i in range(s)]
    rows = np.full((p, 3 + 9 * s), 0xEE, np.uint8)
    orc.allgatherv(dims, offsets, one, 7, rows, gd)
    ref = orc.allgather(dims, offsets, one)
    for i in range(s):
        assert np.array_equal(rows[:, gd[i]:gd[i] + 7], ref[:, i])
    # the paper's worked sizes for base 512 in three dimensions
    big = gen.stencil_block_sizes(offsets, 512)
    assert sorted(set(big)) == _ints(golden["irregular_d3_base512_sizes"])
    assert abs(sum(big) / 1e6 - float(golden["irregular_d3_base512_total_MB"])) < 0.1
    assert (big.count(262144), big.count(512), big.count(1)) == (6, 12, 8)


# ---------------------------------------------------------------- meshes

MESHES = [
    ((5,), (0,), [(1,), (-2,), (7,), (0,)]),
    ((4, 3), (0, 0), gen.moore(2, 1)),
    ((4, 3), (1, 0), gen.moore(2, 1) + [(0, 0), (5, 1)]),
    ((3, 4, 2), (0, 1, 0), gen.moore(3, 1)),
    ((6, 5), (0, 0), gen.von_neumann(2, 2)),
]


@pytest.mark.parametrize("dims,periodic,offsets", MESHES)
def test_mesh_definition_by_slicing_and_by_push(dims, periodic, offsets):
    p, s, d = int(np.prod(dims)), len(offsets), len(dims)
    send = _rand_send(p, s, 3)
    recv = orc.alltoall_mesh(dims, periodic, offsets, send, np.full_like(send, 0xEE))
    # (a) array slicing: in a non-periodic dimension the receiving coordinates are
    # [max(0,c), min(p, p+c)) and read from the same range moved back by c
    for i, C in enumerate(offsets):
        grid = send[:, i].reshape(tuple(dims) + (3,))
        want = np.full_like(grid, 0xEE)
        rolled = grid
        dst_sl, src_sl = [], []
        for j in range(d):
            if periodic[j]:
                rolled = np.roll(rolled, C[j], axis=j)
                dst_sl.append(slice(None)); src_sl.append(slice(None))
            else:
                lo, hi = max(0, C[j]), min(dims[j], dims[j] + C[j])
                dst_sl.append(slice(lo, max(lo, hi))); src_sl.append(slice(lo - C[j], max(lo, hi) - C[j]))
        want[tuple(dst_sl)] = rolled[tuple(src_sl)]
        assert np.array_equal(recv[:, i].reshape(want.shape), want), (i, C)
    # (b) pure-Python push: every process hands block i to R + C^i if that process exists
    coords = list(itertools.product(*[range(n) for n in dims]))
    index = {c: r for r, c in enumerate(coords)}
    want = [[None] * s for _ in coords]
    for R, rc in enumerate(coords):
        for i, C in enumerate(offsets):
            t = tuple((rc[j] + C[j]) % dims[j] if periodic[j] else rc[j] + C[j] for j in range(d))
            if t in index:
                want[index[t]][i] = send[R, i]
    for R in range(p):
        for i in range(s):
            exp = want[R][i] if want[R][i] is not None else np.full(3, 0xEE, np.uint8)
            assert np.array_equal(recv[R, i], exp), (R, i)
    one = np.ascontiguousarray(send[:, 0])
    rep = np.repeat(one[:, None, :], s, axis=1)
    assert np.array_equal(orc.allgather_mesh(dims, periodic, offsets, one, np.full_like(send, 0xEE)),
                          orc.alltoall_mesh(dims, periodic, offsets, rep, np.full_like(send, 0xEE)))


def test_fully_periodic_mesh_is_the_torus():
    dims, offsets = (4, 3, 5), gen.moore(3, 1)
    send = _rand_send(60, 26, 2)
    got = orc.alltoall_mesh(dims, (1, 1, 1), offsets, send, np.zeros_like(send))
    assert np.array_equal(got, orc.alltoall(dims, offsets, send))
