"""GPU parity of the slot-major buffer layout ([s][p][m]: one plane of p blocks per
neighbour) against the CPU oracle, bit for bit.  The oracle works on the paper's
[p][s][m] layout; the expected slot-major buffer is the oracle's result with its two
leading indices swapped."""
import numpy as np
import pytest
import torch

import iso_inputs as gen
import paper_1606_07676_amd as iso
from oracle import iso_oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
SM = iso.ISO_LAYOUT_SLOT_MAJOR
ALGS = [iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_BYDIM, iso.ISO_ALG_SX_ROUNDS, iso.ISO_ALG_SX_FUSED,
        iso.ISO_ALG_ONEHOP]
ALG_NAMES = {0: "combined", 1: "combined_bydim", 2: "sx_rounds", 3: "sx_fused", 4: "onehop"}

CASES = [
    ((5,), [(1,), (-2,), (7,)]),
    ((4, 3), [(1, 0), (0, -1), (1, 1), (-1, 2), (0, 0), (1, 1)]),
    ((3, 2, 4), gen.moore(3, 1)),
    ((2, 2, 2, 2), gen.moore(4, 1)),                      # s = 80 > p = 16
    ((9, 9, 9), [(0, 0, 0), (0, 0, 1), (1, 0, 0), (1, 1, 0), (1, 1, 1), (3, 2, 0), (3, 3, 2),
                 (4, 0, 1), (4, 0, 2), (4, 1, 1)]),
    ((37, 11), gen.moore(2, 2)),                          # several tiles, ragged tail
    ((2, 2, 2, 2, 2), gen.moore(5, 1)),                   # 162 entries in one round: table too big for LDS
    ((8, 4, 8), gen.moore(3, 3)),                         # s = 342
]
BLOCK_SIZES = [16, 48, 256, 1, 6, 1040]


def _comm(dims, offsets, periodic=None):
    arr = np.asarray(offsets, np.int32).reshape(len(offsets), len(dims))
    return iso.iso_neighborhood_create(dims, arr) if periodic is None else \
        iso.iso_neighborhood_create_mesh(dims, periodic, arr)


def _run(comm, op, alg, m, send, p, s, layout=SM):
    wsb = iso.iso_workspace_bytes(comm, op, alg, m)
    recv = torch.full((s, p, m), 0xEE, dtype=torch.uint8, device=DEV)
    work = torch.full((max(wsb, 16),), 0xDD, dtype=torch.uint8, device=DEV)
    init = iso.iso_neighbor_alltoall_init_layout if op == iso.ISO_OP_ALLTOALL else \
        iso.iso_neighbor_allgather_init_layout
    req = init(send, recv, m, layout, work, comm, alg)
    info = iso.iso_request_info(req)
    iso.iso_start(req)
    iso.iso_wait(req)
    iso.iso_request_free(req)
    return recv, info


@pytest.mark.parametrize("alg", ALGS, ids=lambda a: ALG_NAMES[a])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_slot_major_every_byte(case, alg):
    dims, offsets = CASES[case]
    p, s = int(np.prod(dims)), len(offsets)
    comm = _comm(dims, offsets)
    for m in BLOCK_SIZES:
        send_h = gen.alltoall_send(400 + case, p, s, m)                        # [p][s][m]
        want = orc.alltoall(dims, offsets, send_h).transpose(1, 0, 2)          # [s][p][m]
        send = torch.from_numpy(np.ascontiguousarray(send_h.transpose(1, 0, 2))).to(DEV)
        keep = send.clone()
        recv, info = _run(comm, iso.ISO_OP_ALLTOALL, alg, m, send, p, s)
        assert np.array_equal(recv.cpu().numpy(), want), f"a2a dims={dims} m={m} alg={alg}"
        assert torch.equal(send, keep), "send buffer was modified"
        assert info["delivered_bytes"] == p * s * m
        one_h = gen.allgather_send(400 + case, p, m)
        wantg = orc.allgather(dims, offsets, one_h).transpose(1, 0, 2)
        recv, _ = _run(comm, iso.ISO_OP_ALLGATHER, alg, m, torch.from_numpy(one_h).to(DEV), p, s)
        assert np.array_equal(recv.cpu().numpy(), wantg), f"ag dims={dims} m={m} alg={alg}"


def test_slot_major_on_a_mesh_and_layout_argument():
    dims, periodic, offsets, m = (6, 5, 4), (0, 1, 0), gen.moore(3, 1), 48
    p, s = 120, 26
    comm = _comm(dims, offsets, periodic)
    send_h = gen.alltoall_send(9, p, s, m)
    want = orc.alltoall_mesh(dims, periodic, offsets, send_h, np.full((p, s, m), 0xEE, np.uint8))
    send = torch.from_numpy(np.ascontiguousarray(send_h.transpose(1, 0, 2))).to(DEV)
    for alg in ALGS[:4]:
        recv, _ = _run(comm, iso.ISO_OP_ALLTOALL, alg, m, send, p, s)
        assert np.array_equal(recv.cpu().numpy(), want.transpose(1, 0, 2)), ALG_NAMES[alg]
    # ISO_LAYOUT_RANK_MAJOR through the same call is the plain call
    torus = _comm(dims, offsets)
    rm = torch.from_numpy(send_h).to(DEV)
    recv, _ = _run(torus, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, m, rm, p, s, layout=iso.ISO_LAYOUT_RANK_MAJOR)
    assert np.array_equal(recv.cpu().numpy().reshape(p, s, m), orc.alltoall(dims, offsets, send_h))
    with pytest.raises(iso.IsoError) as e:
        _run(torus, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, m, rm, p, s, layout=7)
    assert e.value.status == iso.ISO_ERR_ARG


@pytest.mark.parametrize("key,m", [(2, 256), (4, 16), (3, 1024)])
def test_slot_major_named_workloads_full_size(key, m):
    """Full size, message-combining schedule: every received plane against the block the
    generator gives for the oracle's source rank."""
    cfg = gen.get_config(key)
    p, s = cfg.p, cfg.s
    comm = _comm(cfg.dims, cfg.offsets)
    src = torch.from_numpy(orc.source_ranks(cfg.dims, cfg.offsets)).to(DEV)          # (p, s) from the oracle
    ranks = torch.arange(p, device=DEV)
    seed = 7000 + key
    for op_name in cfg.ops:
        if op_name == "alltoall":
            send = torch.empty((s, p, m), dtype=torch.uint8, device=DEV)
            for i in range(s):
                send[i] = gen.block_bytes_torch(seed, ranks, torch.full_like(ranks, i), m, cfg.kind)
            recv, info = _run(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, m, send, p, s)
            for i in range(s):
                want = gen.block_bytes_torch(seed, src[:, i], torch.full_like(ranks, i), m, cfg.kind)
                assert torch.equal(recv[i], want), f"{cfg.name} a2a plane {i}"
        else:
            send = gen.allgather_send_torch(seed, p, m, cfg.kind, device=DEV)
            recv, info = _run(comm, iso.ISO_OP_ALLGATHER, iso.ISO_ALG_COMBINED, m, send, p, s)
            for i in range(s):
                want = gen.block_bytes_torch(seed ^ gen.ALLGATHER_TWEAK, src[:, i], torch.zeros_like(ranks), m,
                                             cfg.kind)
                assert torch.equal(recv[i], want), f"{cfg.name} ag plane {i}"
        assert info["vector_bytes"] == 16
