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
        iso.ISO_ALG_ONEHOP, iso.ISO_ALG_COMBINED_STAGED]
ALG_NAMES = {0: "combined", 1: "combined_bydim", 2: "sx_rounds", 3: "sx_fused", 4: "onehop", 5: "combined_staged"}

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
    ((7, 5, 6), gen.positive_octant(3, 3)),               # s = 63, asymmetric
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


@pytest.mark.parametrize("alg", [iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_BYDIM, iso.ISO_ALG_ONEHOP],
                         ids=lambda a: ALG_NAMES[a])
def test_slot_major_shales_neighbourhood(alg):
    """Section 6's 1396-neighbour shells on a 9 x 8 x 8 torus: 1396 planes, launches with several
    hundred entries."""
    dims, offsets, m = (9, 8, 8), gen.shales(3, (3, 7)), 16
    p, s = 576, len(offsets)
    comm = _comm(dims, offsets)
    send_h = gen.alltoall_send(31, p, s, m)
    send = torch.from_numpy(np.ascontiguousarray(send_h.transpose(1, 0, 2))).to(DEV)
    recv, _ = _run(comm, iso.ISO_OP_ALLTOALL, alg, m, send, p, s)
    assert np.array_equal(recv.cpu().numpy(), orc.alltoall(dims, offsets, send_h).transpose(1, 0, 2))
    one_h = gen.allgather_send(32, p, m)
    recv, _ = _run(comm, iso.ISO_OP_ALLGATHER, alg, m, torch.from_numpy(one_h).to(DEV), p, s)
    assert np.array_equal(recv.cpu().numpy(), orc.allgather(dims, offsets, one_h).transpose(1, 0, 2))


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


# ---------------------------------------------------------------- irregular blocks, one plane per neighbour

def _planes(sizes, p, align, gap):
    """Start of every plane and the total length: plane i holds p blocks of sizes[i] bytes."""
    displs, at = [], gap
    for sz in sizes:
        at = -(-at // align) * align
        displs.append(at)
        at += p * sz + gap
    return displs, at + 3


IRREGULAR = [
    ((4, 3, 5), gen.moore(3, 1), "stencil"),
    ((6, 5), gen.von_neumann(2, 2), "odd"),
    ((9, 9, 9), CASES[4][1], "odd"),
    ((37, 11), gen.moore(2, 2), "stencil"),
    ((5, 4), [(1, 1), (1, 1), (1, 1), (0, 0), (0, 0), (2, 0), (2, 0)], "odd"),
]


@pytest.mark.parametrize("alg", ALGS, ids=lambda a: ALG_NAMES[a])
@pytest.mark.parametrize("case", range(len(IRREGULAR)))
def test_slot_major_irregular_every_byte(case, alg):
    dims, offsets, flavour = IRREGULAR[case]
    p, s = int(np.prod(dims)), len(offsets)
    rng = np.random.default_rng(900 + case)
    if flavour == "stencil":
        sizes = [(4096, 64, 16, 1)[i % 4] for i in range(s)]
        align, gap = 16, 0
    else:
        sizes = [int(x) for x in rng.integers(1, 40, size=s)]
        sizes[s // 2] = 0
        align, gap = 1, 2
    rm_displ, ext = gen.packed_displacements(sizes, 1)
    send_rm = rng.integers(0, 256, size=(p, max(ext, 1)), dtype=np.uint8)
    want_rm = orc.alltoallv(dims, offsets, send_rm, sizes, rm_displ, np.full_like(send_rm, 0xEE), rm_displ)
    sd, slen = _planes(sizes, p, align, gap)
    rd, rlen = _planes(sizes[::-1], p, align, gap + 1)
    rd = rd[::-1]
    send_h = np.full(slen, 0x11, np.uint8)
    want = np.full(rlen, 0xEE, np.uint8)
    for i, sz in enumerate(sizes):
        send_h[sd[i]:sd[i] + p * sz] = send_rm[:, rm_displ[i]:rm_displ[i] + sz].reshape(-1)
        want[rd[i]:rd[i] + p * sz] = want_rm[:, rm_displ[i]:rm_displ[i] + sz].reshape(-1)
    comm = _comm(dims, offsets)
    send = torch.from_numpy(send_h).to(DEV)
    recv = torch.full((rlen,), 0xEE, dtype=torch.uint8, device=DEV)
    wsb = iso.iso_workspace_bytes_v(comm, iso.ISO_OP_ALLTOALL, alg, sizes)
    work = torch.full((max(wsb, 16),), 0xDD, dtype=torch.uint8, device=DEV)
    req = iso.iso_neighbor_alltoallv_init_layout(send, sizes, sd, 0, recv, sizes, rd, 0, SM, work, comm, alg)
    iso.iso_start(req)
    iso.iso_wait(req)
    iso.iso_request_free(req)
    assert np.array_equal(recv.cpu().numpy(), want), f"dims={dims} {flavour} alg={alg}"
    assert np.array_equal(send.cpu().numpy(), send_h)
    # allgather: every rank contributes one block of m bytes, received into s planes
    m = 48 if flavour == "stencil" else 7
    one = rng.integers(0, 256, size=(p, m + 3), dtype=np.uint8)
    gd_rm = [i * m for i in range(s)]
    wantg_rm = orc.allgatherv(dims, offsets, one, m, np.full((p, max(s * m, 1)), 0xEE, np.uint8), gd_rm)
    gd, glen = _planes([m] * s, p, align, gap)
    wantg = np.full(glen, 0xEE, np.uint8)
    for i in range(s):
        wantg[gd[i]:gd[i] + p * m] = wantg_rm[:, gd_rm[i]:gd_rm[i] + m].reshape(-1)
    grecv = torch.full((glen,), 0xEE, dtype=torch.uint8, device=DEV)
    wsb = iso.iso_workspace_bytes_v(comm, iso.ISO_OP_ALLGATHER, alg, [m] * s)
    gwork = torch.empty(max(wsb, 16), dtype=torch.uint8, device=DEV)
    req = iso.iso_neighbor_allgatherv_init_layout(torch.from_numpy(one).to(DEV), m, m + 3, grecv, [m] * s, gd, 0,
                                                  SM, gwork, comm, alg)
    iso.iso_start(req)
    iso.iso_wait(req)
    iso.iso_request_free(req)
    assert np.array_equal(grecv.cpu().numpy(), wantg), f"allgather dims={dims} alg={alg}"


def test_slot_major_irregular_argument_checks():
    dims, offsets = (4, 3), gen.moore(2, 1)
    p, s = 12, 8
    comm = _comm(dims, offsets)
    sizes = [16] * s
    d, n = _planes(sizes, p, 16, 0)
    buf = torch.zeros(n, dtype=torch.uint8, device=DEV)
    out = torch.zeros(n, dtype=torch.uint8, device=DEV)
    work = torch.zeros(n, dtype=torch.uint8, device=DEV)
    clash = list(d)
    clash[1] = d[0] + 16                      # plane 1 starts inside plane 0
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoallv_init_layout(buf, sizes, d, 0, out, sizes, clash, 0, SM, work, comm)
    assert e.value.status == iso.ISO_ERR_OVERLAP
    req = iso.iso_neighbor_alltoallv_init_layout(buf, sizes, clash, 0, out, sizes, d, 0, SM, work, comm)  # send may
    iso.iso_request_free(req)
    with pytest.raises(iso.IsoError) as e:      # sizes must match pairwise, whatever the layout
        iso.iso_neighbor_alltoallv_init_layout(buf, sizes, d, 0, out, [16] * (s - 1) + [32], d, 0, SM, work, comm)
    assert e.value.status == iso.ISO_ERR_ARG


def test_slot_major_irregular_on_a_mesh():
    dims, periodic, offsets = (9, 7, 5), (0, 0, 1), gen.moore(3, 1)
    p, s = 315, 26
    sizes = gen.stencil_block_sizes(offsets, 16)              # 256 / 16 / 1 bytes
    sd, n = _planes(sizes, p, 16, 0)
    rng = np.random.default_rng(31)
    send_h = rng.integers(0, 256, size=n, dtype=np.uint8)
    src, valid = orc.source_ranks_mesh(dims, periodic, offsets)
    want = np.full(n, 0xEE, np.uint8)
    for i, sz in enumerate(sizes):
        plane_in = send_h[sd[i]:sd[i] + p * sz].reshape(p, sz)
        plane_out = want[sd[i]:sd[i] + p * sz].reshape(p, sz)
        v = valid[:, i]
        plane_out[v] = plane_in[src[v, i]]
    comm = _comm(dims, offsets, periodic)
    send = torch.from_numpy(send_h).to(DEV)
    for alg in ALGS[:4]:
        recv = torch.full((n,), 0xEE, dtype=torch.uint8, device=DEV)
        wsb = iso.iso_workspace_bytes_v(comm, iso.ISO_OP_ALLTOALL, alg, sizes)
        work = torch.empty(max(wsb, 16), dtype=torch.uint8, device=DEV)
        req = iso.iso_neighbor_alltoallv_init_layout(send, sizes, sd, 0, recv, sizes, sd, 0, SM, work, comm, alg)
        iso.iso_start(req)
        iso.iso_wait(req)
        iso.iso_request_free(req)
        assert np.array_equal(recv.cpu().numpy(), want), ALG_NAMES[alg]
