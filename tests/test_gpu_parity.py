"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
bit for bit, on seeded inputs.  Small cases compare every byte with the numpy
oracle; the five named workloads run at full size in the launch configuration
the benchmark times and are compared in rank chunks with what the oracle says
each received block must be (the block generated for the oracle's source rank).
"""
import numpy as np
import pytest
import torch

import iso_inputs as gen
import paper_1606_07676_amd as iso
from oracle import iso_oracle as orc
from oracle import c_twin

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
ALGS = [iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_BYDIM, iso.ISO_ALG_SX_ROUNDS, iso.ISO_ALG_SX_FUSED,
        iso.ISO_ALG_ONEHOP, iso.ISO_ALG_COMBINED_STAGED]
ALG_NAMES = {0: "combined", 1: "combined_bydim", 2: "sx_rounds", 3: "sx_fused", 4: "onehop", 5: "combined_staged"}

SMALL = [
    ((5,), [(1,), (-2,), (7,)]),
    ((4, 3), [(1, 0), (0, -1), (1, 1), (-1, 2), (0, 0), (1, 1)]),
    ((3, 2, 4), gen.moore(3, 1)),
    ((2, 1, 5), [(1, 0, 2), (0, 3, -1), (-5, 0, 6), (0, 0, 0), (2, 7, 5)]),
    ((2, 2, 2, 2), gen.moore(4, 1)),                      # s = 80 > p = 16
    ((6, 5), gen.von_neumann(2, 2)),
    ((9, 9, 9), [(0, 0, 0), (0, 0, 1), (1, 0, 0), (1, 1, 0), (1, 1, 1), (3, 2, 0), (3, 3, 2),
                 (4, 0, 1), (4, 0, 2), (4, 1, 1)]),
    ((4, 4, 4, 4, 4), gen.random_distinct(5, -3, 3, 40, 99)),
    ((5, 4), [(1, 1), (1, 1), (1, 1), (0, 0), (0, 0), (2, 0), (2, 0)]),
    ((37, 11), gen.moore(2, 2)),                          # several tiles, ragged tail
    ((1, 1), [(0, 0), (3, -2)]),                          # a single process
    ((2, 2, 2, 2, 2), gen.moore(5, 1)),                   # 162 entries in one round: table too big for LDS
    ((8, 4, 8), gen.moore(3, 3)),                         # s = 342, radius > 1, wrap-around aliases
    ((7, 5, 6), gen.positive_octant(3, 3)),               # s = 63, the asymmetric neighbourhood of Section 4
]
BLOCK_SIZES = [16, 48, 256, 1, 6, 20, 8, 1040]


def _comm(dims, offsets):
    return iso.iso_neighborhood_create(dims, np.asarray(offsets, np.int32).reshape(len(offsets), len(dims)))


def _run(dims, offsets, op, alg, m, send, misalign=0, stream=None, starts=1):
    """send: device uint8 tensor.  Returns recv (p, s, m) device tensor."""
    p, s = int(np.prod(dims)), len(offsets)
    comm = _comm(dims, offsets)
    wsb = iso.iso_workspace_bytes(comm, op, alg, m)
    recv_store = torch.full((p * s * m + misalign + 16,), 0xEE, dtype=torch.uint8, device=DEV)
    recv = recv_store[misalign:misalign + p * s * m]
    work = torch.full((wsb + 16,), 0xDD, dtype=torch.uint8, device=DEV)[:wsb] if wsb else None
    init = iso.iso_neighbor_alltoall_init if op == iso.ISO_OP_ALLTOALL else iso.iso_neighbor_allgather_init
    req = init(send, recv, m, work, comm, alg)
    info = iso.iso_request_info(req)
    for _ in range(starts):
        iso.iso_start(req, stream)
    iso.iso_wait(req)
    iso.iso_request_free(req)
    return recv.view(p, s, m), info


@pytest.mark.parametrize("alg", ALGS, ids=lambda a: ALG_NAMES[a])
@pytest.mark.parametrize("case", range(len(SMALL)))
def test_small_alltoall_every_byte(case, alg):
    dims, offsets = SMALL[case]
    p, s = int(np.prod(dims)), len(offsets)
    for m in BLOCK_SIZES:
        send_h = gen.alltoall_send(100 + case, p, s, m)
        send = torch.from_numpy(send_h).to(DEV)
        recv, info = _run(dims, offsets, iso.ISO_OP_ALLTOALL, alg, m, send)
        want = orc.alltoall(dims, offsets, send_h)
        assert np.array_equal(recv.cpu().numpy(), want), f"dims={dims} m={m} alg={alg}"
        assert np.array_equal(send.cpu().numpy(), send_h), "send buffer was modified"
        assert info["delivered_bytes"] == p * s * m


@pytest.mark.parametrize("alg", ALGS, ids=lambda a: ALG_NAMES[a])
@pytest.mark.parametrize("case", range(len(SMALL)))
def test_small_allgather_every_byte(case, alg):
    dims, offsets = SMALL[case]
    p = int(np.prod(dims))
    for m in BLOCK_SIZES:
        send_h = gen.allgather_send(200 + case, p, m)
        send = torch.from_numpy(send_h).to(DEV)
        recv, _ = _run(dims, offsets, iso.ISO_OP_ALLGATHER, alg, m, send)
        want = orc.allgather(dims, offsets, send_h)
        assert np.array_equal(recv.cpu().numpy(), want), f"dims={dims} m={m} alg={alg}"


@pytest.mark.parametrize("alg", ALGS, ids=lambda a: ALG_NAMES[a])
@pytest.mark.parametrize("dims", [(15, 16, 17), (9, 8, 8)], ids=["no_alias", "aliased"])
def test_shales_neighbourhood(dims, alg):
    """Section 6's largest neighbourhood: the Chebyshev shells of radius 3 and 7 in three
    dimensions, 1396 neighbours.  Every coordinate value from -7 to 7 occurs, so the
    torus-direct schedule has one round per dimension and non-zero residue (Section 5):
    14 * 3 = 42 on a torus whose sizes exceed 14; on the 9 x 8 x 8 torus (576 processes as
    in the paper's runs) values alias and 8 + 7 + 7 = 22 residues are left.  Rounds hold up
    to several hundred entries (more than the LDS table takes)."""
    offsets = gen.shales(3, (3, 7))
    p, s = int(np.prod(dims)), len(offsets)
    assert s == 1396
    direct_rounds = sum(len({c[j] % dims[j] for c in offsets} - {0}) for j in range(3))
    # one-hop schedule (Section 3.1): per dimension the longest walk up plus the longest walk down,
    # counted on the coordinates as given
    onehop_rounds = sum(max(c[j] for c in offsets) - min(c[j] for c in offsets) for j in range(3))
    # staged schedule: the rounds that keep an entry, then (more than 128 neighbours: no kernel of
    # its own for the last launch) one launch per dimension that some block's last hop runs along
    comm = iso.iso_neighborhood_create(dims, np.asarray(offsets, np.int32))
    plan = iso.iso_plan_create(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED_STAGED)
    n_rounds = iso.iso_plan_info(plan)["launches"]
    staged_launches = n_rounds - 1 + len({e["dim"] for e in iso.iso_plan_entries(plan, n_rounds - 1)})
    for m in (16, 40):
        send_h = gen.alltoall_send(77, p, s, m)
        send = torch.from_numpy(send_h).to(DEV)
        recv, info = _run(dims, offsets, iso.ISO_OP_ALLTOALL, alg, m, send)
        assert np.array_equal(recv.cpu().numpy(), orc.alltoall(dims, offsets, send_h)), f"alltoall m={m}"
        assert info["launches"] == {iso.ISO_ALG_COMBINED: direct_rounds, iso.ISO_ALG_COMBINED_BYDIM: 3,
                                    iso.ISO_ALG_SX_ROUNDS: s, iso.ISO_ALG_SX_FUSED: 1,
                                    iso.ISO_ALG_ONEHOP: onehop_rounds,
                                    iso.ISO_ALG_COMBINED_STAGED: staged_launches}[alg]
        del send, recv
        send_h = gen.allgather_send(78, p, m)
        send = torch.from_numpy(send_h).to(DEV)
        recv, info = _run(dims, offsets, iso.ISO_OP_ALLGATHER, alg, m, send)
        assert np.array_equal(recv.cpu().numpy(), orc.allgather(dims, offsets, send_h)), f"allgather m={m}"
    assert direct_rounds == (42 if dims[0] == 15 else 22) and onehop_rounds == 42


@pytest.mark.parametrize("alg", [iso.ISO_ALG_COMBINED, iso.ISO_ALG_SX_FUSED, iso.ISO_ALG_COMBINED_STAGED],
                         ids=lambda a: ALG_NAMES[a])
@pytest.mark.parametrize("send_off,recv_off", [(0, 0), (8, 8), (8, 0), (4, 12), (2, 2), (1, 1), (1, 2), (3, 0),
                                               (0, 13)])
def test_unaligned_buffers_keep_the_full_unit_width(send_off, recv_off, alg):
    """Buffer addresses need no alignment: blocks of 16 bytes and more move in 16-byte units
    wherever the buffers start, and the bytes around the buffers stay as they were."""
    dims, offsets = (6, 5), gen.moore(2, 1)
    p, s = 30, 8
    for m in (64, 52, 17):
        n = p * s * m
        send_h = gen.alltoall_send(5, p, s, m)
        send_store = torch.full((n + 48,), 0xAB, dtype=torch.uint8, device=DEV)
        send = send_store[16 + send_off:16 + send_off + n]
        send.copy_(torch.from_numpy(send_h.reshape(-1)).to(DEV))
        recv_store = torch.full((n + 48,), 0xEE, dtype=torch.uint8, device=DEV)
        recv = recv_store[16 + recv_off:16 + recv_off + n]
        comm = _comm(dims, offsets)
        wsb = iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, alg, m)
        work = torch.empty(max(wsb, 16), dtype=torch.uint8, device=DEV)
        req = iso.iso_neighbor_alltoall_init(send, recv, m, work, comm, alg)
        assert iso.iso_request_info(req)["vector_bytes"] == 16
        iso.iso_start(req)
        iso.iso_wait(req)
        iso.iso_request_free(req)
        assert np.array_equal(recv.cpu().numpy().reshape(p, s, m), orc.alltoall(dims, offsets, send_h)), (m, alg)
        out = recv_store.cpu().numpy()
        assert (out[:16 + recv_off] == 0xEE).all() and (out[16 + recv_off + n:] == 0xEE).all()
        assert np.array_equal(send.cpu().numpy(), send_h.reshape(-1))


@pytest.mark.parametrize("m,vec", [(1, 1), (2, 2), (3, 2), (4, 4), (5, 4), (7, 4), (8, 8), (9, 8), (15, 8),
                                   (16, 16), (17, 16), (31, 16), (33, 16), (100, 16), (1039, 16)])
def test_unit_width_follows_the_block_size(m, vec):
    """The unit is the largest power of two up to 16 bytes that fits the block; a block whose
    size is not a multiple of it ends with a unit that overlaps the one before."""
    dims, offsets = (37, 11), gen.moore(2, 2)
    p, s = 407, 24
    send_h = gen.alltoall_send(6, p, s, m)
    send = torch.from_numpy(send_h).to(DEV)
    for alg in ALGS:
        recv, info = _run(dims, offsets, iso.ISO_OP_ALLTOALL, alg, m, send)
        assert info["vector_bytes"] == vec
        assert np.array_equal(recv.cpu().numpy(), orc.alltoall(dims, offsets, send_h)), (m, alg)
    one_h = gen.allgather_send(7, p, m)
    for alg in ALGS:
        recv, info = _run(dims, offsets, iso.ISO_OP_ALLGATHER, alg, m, torch.from_numpy(one_h).to(DEV))
        assert np.array_equal(recv.cpu().numpy(), orc.allgather(dims, offsets, one_h)), (m, alg)


def test_restart_and_side_stream_give_the_same_result():
    cfg = gen.get_config(1)
    send_h = gen.alltoall_send(3, cfg.p, cfg.s, cfg.m)
    send = torch.from_numpy(send_h).to(DEV)
    want = orc.alltoall(cfg.dims, cfg.offsets, send_h)
    side = torch.cuda.Stream()
    for alg in ALGS:
        recv, info = _run(cfg.dims, cfg.offsets, iso.ISO_OP_ALLTOALL, alg, cfg.m, send, stream=side, starts=3)
        assert np.array_equal(recv.cpu().numpy(), want)
        assert info["launches"] == {iso.ISO_ALG_COMBINED: 4, iso.ISO_ALG_COMBINED_BYDIM: 2,
                                    iso.ISO_ALG_SX_ROUNDS: 8, iso.ISO_ALG_SX_FUSED: 1,
                                    iso.ISO_ALG_ONEHOP: 4, iso.ISO_ALG_COMBINED_STAGED: 2}[alg]


@pytest.mark.parametrize("alg", [iso.ISO_ALG_COMBINED, iso.ISO_ALG_ONEHOP, iso.ISO_ALG_SX_ROUNDS,
                                 iso.ISO_ALG_COMBINED_STAGED], ids=lambda a: ALG_NAMES[a])
def test_graph_replay_matches_eager_every_time(alg):
    """The request's graph (both forms) is replayed several times, with eager work of this
    program (fills, another eager collective) and synchronisations in between; every
    replay must give the oracle's result."""
    cases = [((8, 8), gen.moore(2, 1), 32, iso.ISO_OP_ALLTOALL),
             ((9, 9, 9), SMALL[6][1], 48, iso.ISO_OP_ALLGATHER),
             ((37, 11), gen.moore(2, 2), 256, iso.ISO_OP_ALLTOALL)]
    side = torch.cuda.Stream()
    for dims, offsets, m, op in cases:
        p, s = int(np.prod(dims)), len(offsets)
        comm = _comm(dims, offsets)
        if op == iso.ISO_OP_ALLTOALL:
            send_h = gen.alltoall_send(9, p, s, m)
            want = orc.alltoall(dims, offsets, send_h)
            init = iso.iso_neighbor_alltoall_init
        else:
            send_h = gen.allgather_send(9, p, m)
            want = orc.allgather(dims, offsets, send_h)
            init = iso.iso_neighbor_allgather_init
        send = torch.from_numpy(send_h).to(DEV)
        wsb = iso.iso_workspace_bytes(comm, op, alg, m)
        recv = torch.empty((p, s, m), dtype=torch.uint8, device=DEV)
        work = torch.empty(max(wsb, 16), dtype=torch.uint8, device=DEV)
        req = init(send, recv, m, work, comm, alg)
        for rep in range(6):
            # replays 0-2 as a chain of kernel nodes, 3-5 with the rounds of a dimension as parallel branches
            iso.iso_request_set_graph(req, iso.ISO_GRAPH_CHAIN if rep < 3 else iso.ISO_GRAPH_BRANCHES)
            recv.fill_(0xEE)                       # eager work between replays
            work.fill_(0xDD)
            other, _ = _run(dims, offsets, op, iso.ISO_ALG_SX_FUSED, m, send)     # an eager collective
            torch.cuda.synchronize()
            iso.iso_start(req, side if rep % 2 else None)
            iso.iso_wait(req)
            got = recv.cpu().numpy()
            assert np.array_equal(got, want), f"replay {rep} dims={dims}"
            assert np.array_equal(other.cpu().numpy(), want)
        iso.iso_request_set_graph(req, False)      # and back to individual launches
        recv.fill_(0)
        torch.cuda.synchronize()
        iso.iso_start(req)
        iso.iso_wait(req)
        assert np.array_equal(recv.cpu().numpy(), want)
        iso.iso_request_free(req)


def test_noop_and_error_paths():
    comm = _comm((4, 4), gen.moore(2, 1))
    p, s, m = 16, 8, 32
    send = torch.zeros(p * s * m, dtype=torch.uint8, device=DEV)
    recv = torch.zeros(p * s * m, dtype=torch.uint8, device=DEV)
    work = torch.zeros(p * s * m, dtype=torch.uint8, device=DEV)
    # m == 0: success, no launches
    req = iso.iso_neighbor_alltoall_init(send, recv, 0, None, comm)
    assert iso.iso_request_info(req)["launches"] == 0
    iso.iso_start(req)
    iso.iso_wait(req)
    # s == 0
    empty = iso.iso_neighborhood_create((4, 4), np.zeros((0, 2), np.int32))
    req = iso.iso_neighbor_allgather_init(None, None, 64, None, empty)
    iso.iso_start(req)
    iso.iso_wait(req)
    # overlap
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoall_init(send, send[16:], m, work, comm, workspace_bytes=work.numel())
    assert e.value.status in (iso.ISO_ERR_OVERLAP, iso.ISO_ERR_POINTER)
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoall_init(send, send, m, work, comm)
    assert e.value.status == iso.ISO_ERR_OVERLAP
    # workspace too small / missing
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoall_init(send, recv, m, work[:64], comm)
    assert e.value.status == iso.ISO_ERR_WORKSPACE
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoall_init(send, recv, m, None, comm)
    assert e.value.status == iso.ISO_ERR_WORKSPACE
    # a host pointer is refused before any kernel sees it
    host = np.zeros(p * s * m, np.uint8)
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoall_init(host.ctypes.data, recv, m, work, comm)
    assert e.value.status == iso.ISO_ERR_POINTER
    # a device buffer whose allocation is too short for p*s*m (64 KiB blocks: 8 MiB needed,
    # while a 64-byte tensor sits in a 2 MiB allocator segment)
    big_m = 65536
    big_send = torch.zeros(p * s * big_m, dtype=torch.uint8, device=DEV)
    small = torch.zeros(64, dtype=torch.uint8, device=DEV)
    fused = iso.ISO_ALG_SX_FUSED
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoall_init(big_send, small.data_ptr(), big_m, None, comm, fused)
    assert e.value.status == iso.ISO_ERR_POINTER


def test_copy_reference_copies():
    n = (1 << 22) + 48
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device=DEV)
    dst = torch.zeros(n, dtype=torch.uint8, device=DEV)
    iso.iso_copy_reference(src, dst, n)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    dst.zero_()
    iso.iso_copy_reference(src[1:], dst[1:], n - 1)       # unaligned: narrow path
    torch.cuda.synchronize()
    assert torch.equal(src[1:], dst[1:]) and int(dst[0]) == 0


# ---------------------------------------------------------------- named workloads, full size

def _check_full(cfg, op, alg, m, seed, host_oracle):
    """Run one collective at full size and compare all of recv, in rank chunks,
    with the block the generator gives for the oracle's source rank."""
    p, s = cfg.p, cfg.s
    if op == iso.ISO_OP_ALLTOALL:
        send = gen.alltoall_send_torch(seed, p, s, m, cfg.kind, device=DEV)
    else:
        send = gen.allgather_send_torch(seed, p, m, cfg.kind, device=DEV)
    keep = send.clone() if send.numel() <= (1 << 30) else None
    recv, info = _run(cfg.dims, cfg.offsets, op, alg, m, send)
    assert info["vector_bytes"] == 16
    src = orc.source_ranks(cfg.dims, cfg.offsets)                 # (p, s) from the oracle
    slots = torch.arange(s, device=DEV)[None, :]
    chunk = max(1, (256 << 20) // (s * m))
    for lo in range(0, p, chunk):
        hi = min(p, lo + chunk)
        sr = torch.from_numpy(src[lo:hi]).to(DEV)
        if op == iso.ISO_OP_ALLTOALL:
            want = gen.block_bytes_torch(seed, sr, slots, m, cfg.kind)
        else:
            want = gen.block_bytes_torch(seed ^ gen.ALLGATHER_TWEAK, sr, torch.zeros_like(sr), m, cfg.kind)
        assert torch.equal(recv[lo:hi], want), f"{cfg.name} op={op} alg={alg} ranks {lo}:{hi}"
    if keep is not None:
        assert torch.equal(send, keep), "send buffer was modified"
    if host_oracle:
        # the same comparison against the oracle run on the host buffer, every byte
        send_h = send.cpu().numpy()
        fn = c_twin.alltoall if op == iso.ISO_OP_ALLTOALL else c_twin.allgather
        want_h, _ = fn(cfg.dims, cfg.offsets, send_h)
        assert np.array_equal(recv.cpu().numpy(), want_h)
    return info


def _ops(cfg):
    return [iso.ISO_OP_ALLTOALL if o == "alltoall" else iso.ISO_OP_ALLGATHER for o in cfg.ops]


@pytest.mark.parametrize("alg", ALGS, ids=lambda a: ALG_NAMES[a])
@pytest.mark.parametrize("key", [1, 2, 3, 4])
def test_named_workloads_full_size(key, alg):
    cfg = gen.get_config(key)
    for op in _ops(cfg):
        for m in (cfg.m_sweep or (cfg.m,)):
            info = _check_full(cfg, op, alg, m, seed=key * 1000 + m,
                               host_oracle=(alg == iso.ISO_ALG_COMBINED and m == cfg.m))
            if alg == iso.ISO_ALG_COMBINED:
                want_rounds = len(orc.direct_rounds(cfg.dims, cfg.offsets))
                assert info["launches"] == want_rounds
                moves = (orc.direct_alltoall_volume(cfg.dims, cfg.offsets) if op == iso.ISO_OP_ALLTOALL
                         else orc.direct_allgather_volume(cfg.dims, cfg.offsets))
                assert info["bytes_read"] == moves * cfg.p * m == info["bytes_written"]
            if alg == iso.ISO_ALG_COMBINED_STAGED and op == iso.ISO_OP_ALLTOALL:
                # the combined schedule's moves, regrouped: not a byte more
                assert info["bytes_read"] == orc.direct_alltoall_volume(cfg.dims, cfg.offsets) * cfg.p * m
                assert info["launches"] < len(orc.direct_rounds(cfg.dims, cfg.offsets)) or cfg.d == 1
            if alg == iso.ISO_ALG_ONEHOP:
                assert info["launches"] == orc.onehop_rounds(cfg.offsets)
                if op == iso.ISO_OP_ALLTOALL:
                    assert info["bytes_read"] == orc.onehop_alltoall_volume(cfg.offsets) * cfg.p * m
    # a second seed on the combined path
    if alg == iso.ISO_ALG_COMBINED:
        _check_full(cfg, _ops(cfg)[0], alg, cfg.m, seed=77 + key, host_oracle=False)


def test_round_is_split_when_the_unit_index_would_overflow():
    """Two blocks of 8 MiB + 8 bytes per rank on 4096 ranks, both moved in the single round of
    this neighbourhood: 2 * 4096 * 524289 units of 16 bytes, more than a launch's 32-bit unit
    index holds, so the binding must split the round over two launches.  64 GiB per buffer;
    the last unit of every block overlaps the one before it."""
    dims, offsets, m, seed = (64, 64), [(1, 0), (1, 0)], (8 << 20) + 8, 31
    p, s = 4096, 2
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 2 * p * s * m + (8 << 30):
        pytest.skip("needs 136 GiB of free device memory")
    send = gen.alltoall_send_torch(seed, p, s, m, device=DEV, rank_chunk=4)
    recv, info = _run(dims, offsets, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, m, send)
    assert info["vector_bytes"] == 16
    assert info["launches"] == 2                # 1 round, one entry per launch
    src = orc.source_ranks(dims, offsets)
    slots = torch.arange(s, device=DEV)[None, :]
    chunk = 8
    for lo in range(0, p, chunk):
        hi = min(p, lo + chunk)
        want = gen.block_bytes_torch(seed, torch.from_numpy(src[lo:hi]).to(DEV), slots, m)
        assert torch.equal(recv[lo:hi], want), f"ranks {lo}:{hi}"
    del send, recv, want
    torch.cuda.empty_cache()


@pytest.mark.parametrize("alg", ALGS, ids=lambda a: ALG_NAMES[a])
def test_config5_full_size(alg):
    cfg = gen.get_config(5)
    for op in _ops(cfg):
        info = _check_full(cfg, op, alg, cfg.m, seed=5005, host_oracle=False)
        torch.cuda.empty_cache()
    assert info["delivered_bytes"] == cfg.p * cfg.s * cfg.m


@pytest.mark.parametrize("mode", [iso.ISO_SX_LAUNCHES, iso.ISO_SX_FUSED])
def test_sx_init_calls_are_the_straightforward_algorithm(mode):
    """iso_neighbor_{alltoall,allgather}_sx_init: s launches or one, no workspace, the oracle's bytes."""
    dims, offsets, m = (7, 5, 6), gen.positive_octant(3, 3), 48
    p, s = int(np.prod(dims)), len(offsets)
    comm = _comm(dims, offsets)
    a2a_h, ag_h = gen.alltoall_send(31, p, s, m), gen.allgather_send(31, p, m)
    for init, send_h, want in ((iso.iso_neighbor_alltoall_sx_init, a2a_h, orc.alltoall(dims, offsets, a2a_h)),
                               (iso.iso_neighbor_allgather_sx_init, ag_h, orc.allgather(dims, offsets, ag_h))):
        send = torch.from_numpy(send_h).to(DEV)
        recv = torch.full((p, s, m), 0xEE, dtype=torch.uint8, device=DEV)
        req = init(send, recv, m, mode, comm)
        info = iso.iso_request_info(req)
        assert info["launches"] == (s if mode == iso.ISO_SX_LAUNCHES else 1) and info["workspace_bytes"] == 0
        assert info["algorithm"] == (iso.ISO_ALG_SX_ROUNDS if mode == iso.ISO_SX_LAUNCHES else iso.ISO_ALG_SX_FUSED)
        iso.iso_start(req)
        iso.iso_request_free(req)                  # waits for the collective before it frees the table
        assert np.array_equal(recv.cpu().numpy(), want)
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoall_sx_init(send, recv, m, 7, comm)
    assert e.value.status == iso.ISO_ERR_ARG


@pytest.mark.parametrize("s,m", [(128, 256), (128, 16), (127, 256), (129, 16), (26, 1264), (26, 1248), (5, 6560), (1, 32768),
                                 (1, 32784), (64, 256), (65, 256), (1, 16384), (1, 16400)])
def test_staged_schedule_at_the_limits_of_its_tiles(s, m):
    """The staged schedule's own kernels take up to 128 neighbours and rows of up to 2048 units of 16 bytes
    (one tile; rows of up to 1024 units use a smaller tile); one more neighbour or unit and the same plan
    runs on the general kernels.  Both sides of these limits, on a torus whose rank count (105) is no multiple of any tile's rank count, against the
    oracle, every byte; and a single process."""
    for dims in ((7, 5, 3), (1, 1, 1)):
        p = int(np.prod(dims))
        offsets = gen.random_distinct(3, -3, 3, min(s, 300), 7 + s)[:s] if s > 1 else [(1, 2, 0)]
        while len(offsets) < s:                           # fewer distinct vectors than asked for: repeat some
            offsets = offsets + offsets[:s - len(offsets)]
        send_h = gen.alltoall_send(11, p, s, m)
        recv, info = _run(dims, offsets, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED_STAGED, m, torch.from_numpy(send_h).to(DEV))
        assert np.array_equal(recv.cpu().numpy(), orc.alltoall(dims, offsets, send_h)), (dims, s, m)
        one_h = gen.allgather_send(12, p, m)
        recv, info = _run(dims, offsets, iso.ISO_OP_ALLGATHER, iso.ISO_ALG_COMBINED_STAGED, m, torch.from_numpy(one_h).to(DEV))
        assert np.array_equal(recv.cpu().numpy(), orc.allgather(dims, offsets, one_h)), (dims, s, m)


def test_requests_in_flight_together_on_several_streams():
    """Persistent requests share nothing: eight of them (different tori, algorithms and collectives), each
    started five times in turn on a stream of its own with no synchronisation in between, give the
    oracle's bytes."""
    shapes = [((8, 8), gen.moore(2, 1), 32), ((6, 5, 7), gen.moore(3, 1), 16), ((37, 11), gen.moore(2, 2), 48),
              ((4, 4, 4, 4), gen.von_neumann(4, 1), 272)]
    algs = [iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_STAGED, iso.ISO_ALG_COMBINED_BYDIM, iso.ISO_ALG_SX_FUSED]
    live = []
    for q, (dims, offsets, m) in enumerate(shapes):
        p, s = int(np.prod(dims)), len(offsets)
        comm = _comm(dims, offsets)
        for op in (iso.ISO_OP_ALLTOALL, iso.ISO_OP_ALLGATHER):
            alg = algs[(q + op) % len(algs)]
            if op == iso.ISO_OP_ALLTOALL:
                send_h = gen.alltoall_send(40 + q, p, s, m)
                want = orc.alltoall(dims, offsets, send_h)
                init = iso.iso_neighbor_alltoall_init
            else:
                send_h = gen.allgather_send(40 + q, p, m)
                want = orc.allgather(dims, offsets, send_h)
                init = iso.iso_neighbor_allgather_init
            send = torch.from_numpy(send_h).to(DEV)
            recv = torch.full((p, s, m), 0xEE, dtype=torch.uint8, device=DEV)
            wsb = iso.iso_workspace_bytes(comm, op, alg, m)
            work = torch.empty(max(wsb, 16), dtype=torch.uint8, device=DEV)
            live.append((init(send, recv, m, work, comm, alg), torch.cuda.Stream(), send, recv, work, want, (dims, op, alg)))
    torch.cuda.synchronize()
    for _ in range(5):
        for req, stream, *_ in live:
            iso.iso_start(req, stream)
    for req, stream, send, recv, work, want, what in live:
        iso.iso_wait(req)
        assert np.array_equal(recv.cpu().numpy(), want), what
        iso.iso_request_free(req)


@pytest.mark.parametrize("alg", [iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_BYDIM, iso.ISO_ALG_ONEHOP, iso.ISO_ALG_COMBINED_STAGED],
                         ids=lambda a: ALG_NAMES[a])
@pytest.mark.parametrize("dims,m", [((7, 5, 3), 4096), ((37, 11), 4100), ((64,), 8192), ((5, 13), 4097), ((3, 3, 7), 16384),
                                    ((7, 5, 3), 2048), ((37, 11), 3072), ((13, 5), 2064)])
def test_large_blocks_are_taken_in_groups_of_ranks(dims, m, alg):
    """Blocks of 2 KiB and more on rank-major buffers: the round kernels (the general one, and the one
    for blocks of whole wavefronts at 2 and 3 KiB) walk the ranks in groups of 64 (inside a group entry
    after entry).  Rank counts that are no multiple of 64 (a last partial group),
    exactly 64 and below 64; block sizes with and without an overlapping last unit; every byte."""
    offsets = gen.moore(len(dims), 1) + [(0,) * len(dims)]
    p, s = int(np.prod(dims)), len(offsets)
    send_h = gen.alltoall_send(21, p, s, m)
    recv, info = _run(dims, offsets, iso.ISO_OP_ALLTOALL, alg, m, torch.from_numpy(send_h).to(DEV))
    assert np.array_equal(recv.cpu().numpy(), orc.alltoall(dims, offsets, send_h))
    one_h = gen.allgather_send(22, p, m)
    recv, info = _run(dims, offsets, iso.ISO_OP_ALLGATHER, alg, m, torch.from_numpy(one_h).to(DEV))
    assert np.array_equal(recv.cpu().numpy(), orc.allgather(dims, offsets, one_h))
