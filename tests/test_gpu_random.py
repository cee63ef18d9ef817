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
              iso.ISO_ALG_ONEHOP]
MESH_ALGS = TORUS_ALGS[:4]


def _case(rng, mesh):
    d = int(rng.integers(1, 5))
    dims = tuple(int(x) for x in rng.integers(1, 10, size=d))
    s = int(rng.integers(1, 20))
    span = int(rng.integers(1, 6))
    offsets = [tuple(int(x) for x in rng.integers(-span, span + 1, size=d)) for _ in range(s)]
    for _ in range(int(rng.integers(0, 3))):
        offsets.append(offsets[int(rng.integers(0, len(offsets)))])
    if rng.integers(0, 3) == 0:
        offsets.append((0,) * d)
    periodic = tuple(int(x) for x in rng.integers(0, 2, size=d)) if mesh else (1,) * d
    m = int(rng.choice([1, 3, 4, 8, 16, 24, 32, 48, 100, 256, 272, 1024]))
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
    dims, _, offsets, m = _case(rng, mesh=False)
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
    dims, periodic, offsets, m = _case(rng, mesh=True)
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
