"""The allocation-free all-to-all (iso_neighbor_alltoall_noalloc, for callers that cannot
call hipMalloc) against the persistent entry points, through the C ABI: same bytes in the
receive buffer, on two calls in a row that share the library's static scratch array, the
second with a smaller input; and the oracle agrees with both."""
import numpy as np
import pytest
import torch

import iso_inputs as gen
import paper_1606_07676_amd as iso
from oracle import iso_oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda:0"

# (dims, offsets, m): the first fills most of the scratch array (20 of 26 blocks per rank make
# two or more hops: 20 * 4096 * 384 B = 30 MiB of intermediate buffer), the later ones are smaller
# and must not be disturbed by what the earlier calls left behind
CASES = [
    ((16, 16, 16), gen.moore(3, 1), 384),
    ((8, 8), gen.moore(2, 1), 32),
    ((7, 5, 6), gen.positive_octant(3, 3), 20),
    ((4, 4, 4, 4, 4), gen.random_distinct(5, -3, 3, 40, 99), 48),
]


def _persistent(comm, send, p, s, m, alg):
    recv = torch.full((p, s, m), 0xEE, dtype=torch.uint8, device=DEV)
    wsb = iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, alg, m)
    work = torch.empty(max(wsb, 16), dtype=torch.uint8, device=DEV)
    req = iso.iso_neighbor_alltoall_init(send, recv, m, work, comm, alg)
    iso.iso_start(req)
    iso.iso_wait(req)
    iso.iso_request_free(req)
    return recv


@pytest.mark.parametrize("alg", [iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_BYDIM, iso.ISO_ALG_SX_FUSED,
                                 iso.ISO_ALG_ONEHOP, iso.ISO_ALG_COMBINED_STAGED])
def test_noalloc_equals_persistent_calls_in_a_row(alg):
    prepared = []
    for q, (dims, offsets, m) in enumerate(CASES):
        p, s = int(np.prod(dims)), len(offsets)
        comm = iso.iso_neighborhood_create(dims, offsets)
        send_h = gen.alltoall_send(700 + q, p, s, m)
        send = torch.from_numpy(send_h).to(DEV)
        want = _persistent(comm, send, p, s, m, alg)
        recv = torch.full((p, s, m), 0xEE, dtype=torch.uint8, device=DEV)
        prepared.append((dims, offsets, m, comm, send_h, send, want, recv))
    torch.cuda.synchronize()
    # the calls back to back on one stream, no synchronisation in between: each call's table
    # and intermediate blocks overwrite the previous call's in the shared array
    before = torch.cuda.memory_allocated()
    limit = iso.ISO_NOALLOC_SCRATCH_BYTES - iso.ISO_NOALLOC_TABLE_BYTES
    refused = set()
    for q, (dims, offsets, m, comm, send_h, send, want, recv) in enumerate(prepared):
        if iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, alg, m) > limit:
            # (the staged schedule keeps 28 blocks per rank in the workspace on the first case: 42 MiB)
            with pytest.raises(iso.IsoError) as e:
                iso.iso_neighbor_alltoall_noalloc(send, recv, m, comm, alg)
            assert e.value.status == iso.ISO_ERR_SCRATCH
            refused.add(q)
            continue
        iso.iso_neighbor_alltoall_noalloc(send, recv, m, comm, alg)
    assert torch.cuda.memory_allocated() == before
    assert len(refused) <= 1 and (not refused or alg == iso.ISO_ALG_COMBINED_STAGED)
    torch.cuda.synchronize()
    for q, (dims, offsets, m, comm, send_h, send, want, recv) in enumerate(prepared):
        if q in refused:
            assert bool((recv == 0xEE).all()), "a refused call wrote to the receive buffer"
            continue
        assert torch.equal(recv, want), f"dims={dims} m={m} alg={alg}: differs from the persistent call"
        assert np.array_equal(recv.cpu().numpy(), orc.alltoall(dims, offsets, send_h)), f"dims={dims}: oracle"
        assert np.array_equal(send.cpu().numpy(), send_h), "send buffer was modified"


def test_noalloc_limits_and_errors():
    # config 2 needs 160 MiB of intermediate buffer: more than the static array holds
    cfg = gen.get_config(2)
    comm = iso.iso_neighborhood_create(cfg.dims, cfg.offsets)
    assert iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, cfg.m) > \
        iso.ISO_NOALLOC_SCRATCH_BYTES - iso.ISO_NOALLOC_TABLE_BYTES
    send = torch.zeros((cfg.p, cfg.s, cfg.m), dtype=torch.uint8, device=DEV)
    recv = torch.full((cfg.p, cfg.s, cfg.m), 0xEE, dtype=torch.uint8, device=DEV)
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoall_noalloc(send, recv, cfg.m, comm, iso.ISO_ALG_COMBINED)
    assert e.value.status == iso.ISO_ERR_SCRATCH
    torch.cuda.synchronize()
    assert bool((recv == 0xEE).all()), "a refused call must not touch the receive buffer"
    # the s-exchange needs no intermediate buffer: the same workload fits
    send = gen.alltoall_send_torch(5, cfg.p, cfg.s, cfg.m, device=DEV)
    iso.iso_neighbor_alltoall_noalloc(send, recv, cfg.m, comm, iso.ISO_ALG_SX_FUSED)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    sample = np.unique(rng.integers(0, cfg.p, size=256))
    src = torch.from_numpy(orc.source_ranks(cfg.dims, cfg.offsets, sample)).to(DEV)
    want = gen.block_bytes_torch(5, src, torch.arange(cfg.s, device=DEV)[None, :], cfg.m)
    assert torch.equal(recv[torch.from_numpy(sample).to(DEV)], want)
    # a table that does not fit: 3124 neighbours, 12500 block-moves per rank, 48 bytes each
    offs = gen.moore(5, 2)
    big = iso.iso_neighborhood_create((5,) * 5, offs)
    s = len(offs)
    assert 48 * iso.iso_neighborhood_info(big)["alltoall_moves"] > iso.ISO_NOALLOC_TABLE_BYTES
    send = torch.zeros((3125, s, 16), dtype=torch.uint8, device=DEV)
    recv = torch.zeros((3125, s, 16), dtype=torch.uint8, device=DEV)
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoall_noalloc(send, recv, 16, big, iso.ISO_ALG_COMBINED)
    assert e.value.status == iso.ISO_ERR_SCRATCH
    # overlap and null arguments are refused as in the init call
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighbor_alltoall_noalloc(send, send, 16, big, iso.ISO_ALG_SX_FUSED)
    assert e.value.status == iso.ISO_ERR_OVERLAP
    # empty collectives are a successful no-op
    iso.iso_neighbor_alltoall_noalloc(send, recv, 0, big, iso.ISO_ALG_COMBINED)
