"""GPU parity on seeded random cases: random tori and meshes (dimension sizes 1..9,
so offsets alias and wrap), random signed offsets with repeats and zero vectors,
random block sizes (odd ones included), every algorithm, every byte against the
CPU oracle."""
import numpy as np
import pytest
import torch

import iso_inputs as gen
import paper_1606_07676_amd as iso
from oracle import iso_oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TORUS_ALGS = [iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_BYDIM, iso.ISO_ALG_SX_ROUNDS, iso.ISO_ALG_SX_FUSED,
              iso.ISO_ALG_ONEHOP, iso.ISO_ALG_COMBINED_STAGED]
MESH_ALGS = TORUS_ALGS[:4]


def _case(rng, mesh, d=None):
    """d given: a torus or mesh of that many dimensions with sizes 1..3 and at most 4096 ranks
    (more dimensions than the kernels' unrolled coordinate decodes cover)."""
    if d is None:
        d = int(rng.integers(1, 5))
        dims = tuple(int(x) for x in rng.integers(1, 10, size=d))
    else:
        while True:
            dims = tuple(int(x) for x in rng.choice([1, 2, 2, 2, 3], size=d))
            if 64 <= int(np.prod(dims)) <= 4096:
                break
    s = int(rng.integers(1, 20))
    span = int(rng.integers(1, 6))
    offsets = [tuple(int(x) for x in rng.integers(-span, span + 1, size=d)) for _ in range(s)]
    for _ in range(int(rng.integers(0, 3))):
        offsets.append(offsets[int(rng.integers(0, len(offsets)))])
    if rng.integers(0, 3) == 0:
        offsets.append((0,) * d)
    periodic = tuple(int(x) for x in rng.integers(0, 2, size=d)) if mesh else (1,) * d
    m = int(rng.choice([1, 3, 4, 5, 8, 16, 17, 24, 31, 32, 48, 100, 250, 256, 272, 1024]))
    return dims, periodic, offsets, m


def _run(comm, op, alg, m, send, p, s):
    wsb = iso.iso_workspace_bytes(comm, op, alg, m)
    recv = torch.full((p, s, m), 0xEE, dtype=torch.uint8, device=DEV)
    work = torch.full((max(wsb, 16),), 0xDD, dtype=torch.uint8, device=DEV)
    init = iso.iso_neighbor_alltoall_init if op == iso.ISO_OP_ALLTOALL else iso.iso_neighbor_allgather_init
    req = init(send, recv, m, work, comm, alg)
    iso.iso_start(req)
    iso.iso_wait(req)
    iso.iso_request_free(req)
    return recv.cpu().numpy()


@pytest.mark.parametrize("seed", range(24))
def test_random_torus_every_byte(seed):
    rng = np.random.default_rng(5000 + seed)
    _torus_body(seed, *_case(rng, mesh=False))


@pytest.mark.parametrize("d", [7, 8, 11, 16])
def test_many_dimensions_every_byte(d):
    """Tori and meshes with more dimensions than the coordinate decodes are unrolled for (6):
    the run-time-indexed decodes of the s-exchange, mesh and block kernels."""
    for seed in (0, 1):
        rng = np.random.default_rng(8000 + 10 * d + seed)
        _torus_body(seed, *_case(rng, mesh=False, d=d))
        _mesh_body(seed, *_case(rng, mesh=True, d=d))
        _irregular_body(rng, False, *_case(rng, mesh=False, d=d)[:3])
        _irregular_body(rng, True, *_case(rng, mesh=True, d=d)[:3])


def _torus_body(seed, dims, _, offsets, m):
    p, s = int(np.prod(dims)), len(offsets)
    comm = iso.iso_neighborhood_create(dims, np.asarray(offsets, np.int32).reshape(s, len(dims)))
    a2a_h, ag_h = gen.alltoall_send(seed, p, s, m), gen.allgather_send(seed, p, m)
    want_a2a, want_ag = orc.alltoall(dims, offsets, a2a_h), orc.allgather(dims, offsets, ag_h)
    a2a, ag = torch.from_numpy(a2a_h).to(DEV), torch.from_numpy(ag_h).to(DEV)
    for alg in TORUS_ALGS:
        got = _run(comm, iso.ISO_OP_ALLTOALL, alg, m, a2a, p, s)
        assert np.array_equal(got, want_a2a), (dims, offsets, m, alg)
        got = _run(comm, iso.ISO_OP_ALLGATHER, alg, m, ag, p, s)
        assert np.array_equal(got, want_ag), (dims, offsets, m, alg)
    assert np.array_equal(a2a.cpu().numpy(), a2a_h)


@pytest.mark.parametrize("seed", range(16))
def test_random_mesh_every_byte(seed):
    rng = np.random.default_rng(6000 + seed)
    _mesh_body(seed, *_case(rng, mesh=True))


def _mesh_body(seed, dims, periodic, offsets, m):
    p, s = int(np.prod(dims)), len(offsets)
    comm = iso.iso_neighborhood_create_mesh(dims, periodic, np.asarray(offsets, np.int32).reshape(s, len(dims)))
    a2a_h, ag_h = gen.alltoall_send(seed, p, s, m), gen.allgather_send(seed, p, m)
    keep = np.full((p, s, m), 0xEE, np.uint8)
    want_a2a = orc.alltoall_mesh(dims, periodic, offsets, a2a_h, keep.copy())
    want_ag = orc.allgather_mesh(dims, periodic, offsets, ag_h, keep.copy())
    a2a, ag = torch.from_numpy(a2a_h).to(DEV), torch.from_numpy(ag_h).to(DEV)
    for alg in MESH_ALGS:
        got = _run(comm, iso.ISO_OP_ALLTOALL, alg, m, a2a, p, s)
        assert np.array_equal(got, want_a2a), (dims, periodic, offsets, m, alg)
        got = _run(comm, iso.ISO_OP_ALLGATHER, alg, m, ag, p, s)
        assert np.array_equal(got, want_ag), (dims, periodic, offsets, m, alg)


def _random_sizes(rng, s):
    """per-neighbour block sizes: empty, tiny, around the unit width, large"""
    pool = [0, 1, 2, 3, 7, 8, 15, 16, 17, 31, 33, 64, 100, 255, 256, 300]
    return [int(rng.choice(pool)) for _ in range(s)]


def _gapped_displacements(rng, sizes, order):
    """blocks laid out in `order` with random gaps of 0..4 bytes; returns (displs, extent)"""
    displs, at = [0] * len(sizes), int(rng.integers(0, 4))
    for i in order:
        displs[i] = at
        at += sizes[i] + int(rng.integers(0, 5))
    return displs, at + int(rng.integers(0, 4))


@pytest.mark.parametrize("seed", range(16))
def test_random_irregular_every_byte(seed):
    """All-to-allv and allgatherv on random tori (even seeds) and meshes (odd seeds) with random
    per-neighbour sizes and gapped, byte-aligned displacements, rank-major rows and slot-major
    planes; bytes between blocks must stay untouched."""
    rng = np.random.default_rng(7000 + seed)
    mesh = seed % 2 == 1
    dims, periodic, offsets, _ = _case(rng, mesh)
    _irregular_body(rng, mesh, dims, periodic, offsets)


def _irregular_body(rng, mesh, dims, periodic, offsets):
    d, p, s = len(dims), int(np.prod(dims)), len(offsets)
    arr = np.asarray(offsets, np.int32).reshape(s, d)
    comm = iso.iso_neighborhood_create_mesh(dims, periodic, arr) if mesh else iso.iso_neighborhood_create(dims, arr)
    if mesh:
        src, valid = orc.source_ranks_mesh(dims, periodic, offsets)
    else:
        src, valid = orc.source_ranks(dims, offsets), np.ones((p, s), bool)
    sizes = _random_sizes(rng, s)
    sd, sext = _gapped_displacements(rng, sizes, range(s))
    rd, rext = _gapped_displacements(rng, sizes, reversed(range(s)))
    send_h = rng.integers(0, 256, size=(p, sext), dtype=np.uint8)
    want = np.full((p, rext), 0xEE, np.uint8)
    for i in range(s):
        v = valid[:, i]
        want[v, rd[i]:rd[i] + sizes[i]] = send_h[src[v, i], sd[i]:sd[i] + sizes[i]]
    # slot-major: plane i holds block i of all ranks, p * size_i bytes, planes with gaps
    pd, pext = _gapped_displacements(rng, [p * z for z in sizes], range(s))
    psend_h = rng.integers(0, 256, size=pext, dtype=np.uint8)
    pwant = np.full(pext, 0xEE, np.uint8)
    for i in range(s):
        plane = psend_h[pd[i]:pd[i] + p * sizes[i]].reshape(p, sizes[i])
        out = pwant[pd[i]:pd[i] + p * sizes[i]].reshape(p, sizes[i])
        v = valid[:, i]
        out[v] = plane[src[v, i]]
    # allgatherv: one block of g bytes per rank
    g = int(rng.choice([1, 5, 16, 40, 257]))
    one_h = rng.integers(0, 256, size=(p, g + 3), dtype=np.uint8)
    gd, gext = _gapped_displacements(rng, [g] * s, range(s))
    gwant = np.full((p, gext), 0xEE, np.uint8)
    for i in range(s):
        v = valid[:, i]
        gwant[v, gd[i]:gd[i] + g] = one_h[src[v, i], :g]
    send, psend, one = (torch.from_numpy(x).to(DEV) for x in (send_h, psend_h, one_h))
    for alg in (MESH_ALGS if mesh else TORUS_ALGS):
        wsb = iso.iso_workspace_bytes_v(comm, iso.ISO_OP_ALLTOALL, alg, sizes)
        work = torch.full((max(wsb, 16),), 0xDD, dtype=torch.uint8, device=DEV)
        recv = torch.full((p, rext), 0xEE, dtype=torch.uint8, device=DEV)
        req = iso.iso_neighbor_alltoallv_init(send, sizes, sd, sext, recv, sizes, rd, rext, work, comm, alg)
        iso.iso_start(req)
        iso.iso_wait(req)
        iso.iso_request_free(req)
        assert np.array_equal(recv.cpu().numpy(), want), ("rows", dims, periodic, offsets, sizes, alg)
        precv = torch.full((pext,), 0xEE, dtype=torch.uint8, device=DEV)
        req = iso.iso_neighbor_alltoallv_init_layout(psend, sizes, pd, 0, precv, sizes, pd, 0,
                                                     iso.ISO_LAYOUT_SLOT_MAJOR, work, comm, alg)
        iso.iso_start(req)
        iso.iso_wait(req)
        iso.iso_request_free(req)
        assert np.array_equal(precv.cpu().numpy(), pwant), ("planes", dims, periodic, offsets, sizes, alg)
        wsb = iso.iso_workspace_bytes_v(comm, iso.ISO_OP_ALLGATHER, alg, [g] * s)
        work = torch.full((max(wsb, 16),), 0xDD, dtype=torch.uint8, device=DEV)
        grecv = torch.full((p, gext), 0xEE, dtype=torch.uint8, device=DEV)
        req = iso.iso_neighbor_allgatherv_init(one, g, g + 3, grecv, [g] * s, gd, gext, work, comm, alg)
        iso.iso_start(req)
        iso.iso_wait(req)
        iso.iso_request_free(req)
        assert np.array_equal(grecv.cpu().numpy(), gwant), ("allgatherv", dims, periodic, offsets, g, alg)
    assert np.array_equal(send.cpu().numpy(), send_h) and np.array_equal(psend.cpu().numpy(), psend_h)


def test_many_seeded_tori_regular_and_irregular():
    """A broad sweep in one test: 300 seeded tori (half of them with 128 to 20 000 ranks, so that
    rank groups, leftover ranks and many tiles occur), random neighbourhoods, one regular block
    size and one set of irregular sizes each, all six algorithms, both collectives; every byte
    against the oracle."""
    bad = []
    for seed in range(300):
        rng = np.random.default_rng(777000 + seed)
        lo, hi = (128, 20000) if seed % 2 else (2, 5000)
        for _ in range(10000):
            dims = tuple(int(x) for x in rng.integers(1, 17, size=int(rng.integers(1, 6))))
            p = int(np.prod(dims))
            if lo <= p <= hi:
                break
        else:
            raise AssertionError("no torus drawn")
        d = len(dims)
        s = int(rng.integers(1, 20))
        offsets = [tuple(int(x) for x in rng.integers(-4, 5, size=d)) for _ in range(s)]
        comm = iso.iso_neighborhood_create(dims, np.asarray(offsets, np.int32).reshape(s, d))
        m = int(rng.choice([1, 3, 8, 16, 24, 48, 64, 100, 256, 1024, 2048, 4096, 4100]))
        if p * s * m <= 32 << 20:
            send_h = rng.integers(0, 256, size=(p, s, m), dtype=np.uint8)
            one_h = rng.integers(0, 256, size=(p, m), dtype=np.uint8)
            expected = {iso.ISO_OP_ALLTOALL: orc.alltoall(dims, offsets, send_h),
                        iso.ISO_OP_ALLGATHER: orc.allgather(dims, offsets, one_h)}
            source = {iso.ISO_OP_ALLTOALL: torch.from_numpy(send_h).to(DEV),
                      iso.ISO_OP_ALLGATHER: torch.from_numpy(one_h).to(DEV)}
            for alg in TORUS_ALGS:
                for op in (iso.ISO_OP_ALLTOALL, iso.ISO_OP_ALLGATHER):
                    recv = torch.full((p, s, m), 0xEE, dtype=torch.uint8, device=DEV)
                    work = torch.empty(max(iso.iso_workspace_bytes(comm, op, alg, m), 16), dtype=torch.uint8,
                                       device=DEV)
                    init = (iso.iso_neighbor_alltoall_init if op == iso.ISO_OP_ALLTOALL
                            else iso.iso_neighbor_allgather_init)
                    req = init(source[op], recv, m, work, comm, alg)
                    iso.iso_start(req)
                    iso.iso_wait(req)
                    if not np.array_equal(recv.cpu().numpy(), expected[op]):
                        bad.append(("regular", seed, dims, s, m, alg, op))
                    iso.iso_request_free(req)
        sizes = [int(x) for x in rng.choice([0, 1, 2, 5, 8, 16, 17, 33, 64, 100, 1024, 1030, 4096], size=s)]
        sd, at = [], int(rng.integers(0, 9))
        for sz in sizes:
            sd.append(at)
            at += sz + int(rng.integers(0, 20))
        sext = at + 3
        rd, at = [0] * s, 0
        for i in rng.permutation(s):
            rd[int(i)] = at
            at += sizes[int(i)] + int(rng.integers(0, 7))
        rext = at + 1
        if p * max(sext, rext) <= 32 << 20:
            send_h = rng.integers(0, 256, size=(p, sext), dtype=np.uint8)
            want = orc.alltoallv(dims, offsets, send_h, sizes, sd, np.full((p, rext), 0xEE, np.uint8), rd)
            send = torch.from_numpy(send_h).to(DEV)
            for alg in TORUS_ALGS:
                recv = torch.full((p, rext), 0xEE, dtype=torch.uint8, device=DEV)
                work = torch.empty(max(iso.iso_workspace_bytes_v(comm, iso.ISO_OP_ALLTOALL, alg, sizes), 16),
                                   dtype=torch.uint8, device=DEV)
                req = iso.iso_neighbor_alltoallv_init(send, sizes, sd, sext, recv, sizes, rd, rext, work, comm, alg)
                iso.iso_start(req)
                iso.iso_wait(req)
                if not np.array_equal(recv.cpu().numpy(), want):
                    bad.append(("irregular", seed, dims, sizes, alg))
                iso.iso_request_free(req)
    assert not bad, bad[:5]
