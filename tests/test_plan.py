"""Host logic of libiso through the C ABI, no GPU: symbol export, argument
checks, and the schedules (round lists and block index maps) checked against
the oracle's counts and, by replaying the index maps with numpy.roll on host
arrays, against the oracle's results."""
import os
import re
import subprocess
import tempfile

import numpy as np
import pytest

import iso_inputs as gen
import paper_1606_07676_amd as iso
from oracle import iso_oracle as orc
from conftest import ROOT

RNG = np.random.default_rng(7)

CASES = [
    ((5,), [(1,), (-2,), (7,)]),
    ((4, 3), [(1, 0), (0, -1), (1, 1), (-1, 2), (0, 0), (1, 1)]),
    ((3, 2, 4), gen.moore(3, 1)),
    ((2, 1, 5), [(1, 0, 2), (0, 3, -1), (-5, 0, 6), (0, 0, 0), (2, 7, 5)]),
    ((2, 2, 2, 2), gen.moore(4, 1)),
    ((6, 5), gen.von_neumann(2, 2)),
    ((7, 3, 2), gen.positive_octant(3, 3)),
    ((9, 9, 9), [(0, 0, 0), (0, 0, 1), (1, 0, 0), (1, 1, 0), (1, 1, 1), (3, 2, 0), (3, 3, 2),
                 (4, 0, 1), (4, 0, 2), (4, 1, 1)]),
    ((4, 4, 4, 4, 4), gen.random_distinct(5, -3, 3, 40, 99)),
    ((5, 4), [(1, 1), (1, 1), (1, 1), (0, 0), (0, 0), (2, 0), (2, 0)]),     # repeats
    ((3, 3), []),                                                         # empty neighbourhood
]
ALGS = [iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_BYDIM, iso.ISO_ALG_SX_ROUNDS, iso.ISO_ALG_SX_FUSED,
        iso.ISO_ALG_ONEHOP, iso.ISO_ALG_COMBINED_STAGED]


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "iso.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(iso_[a-z_0-9]+)\s*\(", header))
    assert len(declared) >= 19
    lib = iso.load_library()
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in iso.h but not exported"
    out = subprocess.check_output(["nm", "-D", "--defined-only", iso.library_path()], text=True)
    exported = set(re.findall(r" T (iso_[a-z_0-9]+)", out))
    assert declared == exported


def test_error_strings_and_bad_arguments():
    assert iso.iso_error_string(0) == "success"
    for code in range(1, 9):
        assert iso.iso_error_string(code) not in ("success", "unknown status")
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighborhood_create([4, 0], [(1, 1)])
    assert e.value.status == iso.ISO_ERR_ARG
    with pytest.raises(iso.IsoError):
        iso.iso_neighborhood_create([2] * 17, [[1] * 17])
    with pytest.raises(iso.IsoError) as e:
        iso.iso_neighborhood_create([65536, 65536], [(1, 1)])
    assert e.value.status == iso.ISO_ERR_TOO_LARGE
    comm = iso.iso_neighborhood_create([4, 4], [(1, 1)])
    with pytest.raises(iso.IsoError):
        iso.iso_plan_create(comm, 5, iso.ISO_ALG_COMBINED)
    with pytest.raises(iso.IsoError):
        iso.iso_plan_create(comm, iso.ISO_OP_ALLTOALL, 17)
    plan = iso.iso_plan_create(comm, iso.ISO_OP_ALLTOALL)
    with pytest.raises(iso.IsoError):
        iso.iso_plan_round(plan, 99)
    lib = iso.load_library()
    assert lib.iso_neighborhood_create(2, None, 0, None, None) == iso.ISO_ERR_ARG
    assert lib.iso_start(None, None) == iso.ISO_ERR_ARG
    assert lib.iso_wait(None) == iso.ISO_ERR_ARG
    assert lib.iso_request_free(None) == iso.ISO_ERR_ARG
    # init with a null communicator never reaches the device
    import ctypes
    h = ctypes.c_void_p(123)
    assert lib.iso_neighbor_alltoall_init(None, None, 16, None, 0, None, 0, ctypes.byref(h)) == iso.ISO_ERR_ARG
    assert h.value is None


def _plan_rounds(plan):
    n = iso.iso_plan_info(plan)["launches"]
    return [(iso.iso_plan_round(plan, r), iso.iso_plan_entries(plan, r)) for r in range(n)]


@pytest.mark.parametrize("dims,offsets", CASES)
def test_comm_info_matches_oracle_counts(dims, offsets):
    comm = iso.iso_neighborhood_create(dims, offsets) if offsets else \
        iso.iso_neighborhood_create(dims, np.zeros((0, len(dims)), np.int32))
    info = iso.iso_neighborhood_info(comm)
    assert info["p"] == int(np.prod(dims)) and info["s"] == len(offsets) and info["d"] == len(dims)
    assert info["rounds"] == len(orc.direct_rounds(dims, offsets))
    assert info["alltoall_moves"] == orc.direct_alltoall_volume(dims, offsets)
    can = orc.canonical(dims, offsets)
    assert info["self_slots"] == sum(1 for C in can if not any(C))
    # allgather: never more than the identity-order trie, plus one extra copy per repeated offset
    dup_extra = sum(can[:i].count(C) > 0 and any(C) for i, C in enumerate(can))
    assert info["allgather_moves"] <= orc.direct_allgather_volume(dims, offsets) + dup_extra
    assert info["allgather_moves"] <= info["alltoall_moves"]


def _replay(dims, offsets, op, rounds, work_slots, send, m):
    """Apply the plan's index maps to host arrays.  A SHIFT entry is a
    numpy.roll of one slot plane along one axis; all reads of a launch happen
    before its writes (one kernel launch has no internal ordering)."""
    d, s = len(dims), len(offsets)
    p = int(np.prod(dims))
    shape = tuple(dims)
    bufs = {
        iso.ISO_BUF_SEND: send.reshape(shape + ((s, m) if op == iso.ISO_OP_ALLTOALL else (1, m))),
        iso.ISO_BUF_RECV: np.full(shape + (max(s, 1), m), 0xEE, np.uint8),
        iso.ISO_BUF_WORK: np.full(shape + (max(work_slots, 1), m), 0xDD, np.uint8),
    }
    written = set()
    for info, entries in rounds:
        reads, writes, staged = set(), set(), []
        for e in entries:
            src = bufs[e["src_buf"]][..., e["src_slot"], :]
            if info["kind"] == iso.ISO_ROUND_SHIFT:
                assert 0 <= e["shift"] < dims[info["dim"]]      # 0 only on a ring of one process
                data = np.roll(src, e["shift"], axis=info["dim"])
            elif info["kind"] == iso.ISO_ROUND_SELF:
                data = src.copy()
            elif info["kind"] == iso.ISO_ROUND_DELIVER:       # every entry along its own dimension
                assert -1 <= e["dim"] < d and (e["dim"] >= 0 or e["shift"] == 0)
                data = np.roll(src, e["shift"], axis=e["dim"]) if e["dim"] >= 0 else src.copy()
            else:
                data = np.roll(src, tuple(offsets[e["neighbor"]]), axis=tuple(range(d)))
            if info["kind"] != iso.ISO_ROUND_DELIVER:
                assert e["dim"] == info["dim"]
            staged.append((e, data))
            reads.add((e["src_buf"], e["src_slot"]))
            assert (e["dst_buf"], e["dst_slot"]) not in writes, "two entries write one block"
            writes.add((e["dst_buf"], e["dst_slot"]))
            assert e["dst_buf"] != iso.ISO_BUF_SEND, "send buffer must never be written"
            if e["src_buf"] != iso.ISO_BUF_SEND:
                assert (e["src_buf"], e["src_slot"]) in written, "reads a block nobody wrote"
            if e["dst_buf"] == iso.ISO_BUF_WORK:
                assert 0 <= e["dst_slot"] < work_slots
        assert not (reads & writes), "a block is read and written in one launch"
        for e, data in staged:
            bufs[e["dst_buf"]][..., e["dst_slot"], :] = data
            written.add((e["dst_buf"], e["dst_slot"]))
    return bufs[iso.ISO_BUF_RECV].reshape(p, max(s, 1), m)[:, :s], written


def _check_staged_shape(op, dims, offsets, rounds):
    """Staged schedule: the receive buffer is written by the last launch only, block i by entry i, and
    every move of the launches before is a move of one of the combined schedule's rounds (same dimension,
    same distance), the rounds of a dimension in one launch."""
    s = len(offsets)
    if not s:
        assert not rounds
        return
    for info, entries in rounds[:-1]:
        assert entries and info["kind"] in (iso.ISO_ROUND_SHIFT, iso.ISO_ROUND_SELF)
        assert all(e["dst_buf"] == iso.ISO_BUF_WORK and e["src_buf"] != iso.ISO_BUF_RECV for e in entries)
    info, entries = rounds[-1]
    assert info["kind"] == iso.ISO_ROUND_DELIVER and info["dim"] == -1
    assert [(e["dst_buf"], e["dst_slot"]) for e in entries] == [(iso.ISO_BUF_RECV, i) for i in range(s)]
    assert all(e["src_buf"] != iso.ISO_BUF_RECV for e in entries)
    legal = set(orc.direct_rounds(dims, offsets))
    shift_rounds = [(i, es) for i, es in rounds[:-1] if i["kind"] == iso.ISO_ROUND_SHIFT]
    if op == iso.ISO_OP_ALLTOALL:                # one launch per dimension that keeps a move, dimensions ascending
        seen = [i["dim"] for i, es in shift_rounds]
        assert seen == sorted(set(seen))
    for i, es in shift_rounds:
        assert all((i["dim"], e["shift"]) in legal for e in es)
    for e in entries:
        assert e["dim"] < 0 or (e["dim"], e["shift"]) in legal


@pytest.mark.parametrize("alg", ALGS)
@pytest.mark.parametrize("dims,offsets", CASES)
def test_alltoall_plan_reaches_the_oracle_result(dims, offsets, alg):
    p, s, m = int(np.prod(dims)), len(offsets), 3
    comm = iso.iso_neighborhood_create(dims, np.asarray(offsets, np.int32).reshape(s, len(dims)))
    plan = iso.iso_plan_create(comm, iso.ISO_OP_ALLTOALL, alg)
    pinfo = iso.iso_plan_info(plan)
    rounds = _plan_rounds(plan)
    send = RNG.integers(0, 256, size=(p, s, m), dtype=np.uint8)
    keep = send.copy()
    recv, written = _replay(dims, offsets, iso.ISO_OP_ALLTOALL, rounds, pinfo["work_slots"], send, m)
    assert np.array_equal(recv, orc.alltoall(dims, offsets, send))
    assert np.array_equal(send, keep)
    assert {(iso.ISO_BUF_RECV, i) for i in range(s)} <= written
    can = orc.canonical(dims, offsets)
    n_self = sum(1 for C in can if not any(C))
    if alg in (iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_BYDIM):
        assert pinfo["entries"] == orc.direct_alltoall_volume(dims, offsets) + n_self
        assert pinfo["work_slots"] == sum(1 for C in can if sum(1 for c in C if c) >= 2)
        shift_rounds = [r for r in rounds if r[0]["kind"] == iso.ISO_ROUND_SHIFT]
        if alg == iso.ISO_ALG_COMBINED:
            want = orc.direct_rounds(dims, offsets)
            assert [(r[0]["dim"], r[1][0]["shift"]) for r in shift_rounds] == want
            for info, entries in shift_rounds:
                assert len({e["shift"] for e in entries}) == 1
        else:
            assert len(shift_rounds) == len({j for j, _ in orc.direct_rounds(dims, offsets)})
        assert len(rounds) - len(shift_rounds) == (1 if n_self else 0)
    elif alg == iso.ISO_ALG_COMBINED_STAGED:
        # the moves of the combined schedule, each block's last hop in the last launch; a block with three
        # or more hops passes through the receive buffer on its way in that schedule: an extra slot here
        assert pinfo["entries"] == orc.direct_alltoall_volume(dims, offsets) + n_self
        hops = [sum(1 for c in C if c) for C in can]
        assert pinfo["work_slots"] == sum(1 for h in hops if h >= 2) + sum(1 for h in hops if h >= 3)
        _check_staged_shape(iso.ISO_OP_ALLTOALL, dims, offsets, rounds)
    elif alg == iso.ISO_ALG_ONEHOP:
        # Proposition 1: D steps of one hop each, V = sum of 1-norms block-moves (raw coordinates)
        raw_self = sum(1 for C in offsets if not any(C))
        shift_rounds = [r for r in rounds if r[0]["kind"] == iso.ISO_ROUND_SHIFT]
        assert len(shift_rounds) == orc.onehop_rounds(offsets)
        assert pinfo["entries"] == orc.onehop_alltoall_volume(offsets) + raw_self
        assert [(r[0]["dim"]) for r in shift_rounds] == [j for j, _, _ in orc.onehop_steps(offsets)]
        for info, entries in shift_rounds:
            pj = dims[info["dim"]]
            assert {e["shift"] for e in entries} <= {1 % pj, (pj - 1) % pj} and entries
    else:
        assert pinfo["entries"] == s and pinfo["work_slots"] == 0
        assert len(rounds) == (s if alg == iso.ISO_ALG_SX_ROUNDS else min(s, 1))


@pytest.mark.parametrize("alg", ALGS)
@pytest.mark.parametrize("dims,offsets", CASES)
def test_allgather_plan_reaches_the_oracle_result(dims, offsets, alg):
    p, s, m = int(np.prod(dims)), len(offsets), 3
    comm = iso.iso_neighborhood_create(dims, np.asarray(offsets, np.int32).reshape(s, len(dims)))
    plan = iso.iso_plan_create(comm, iso.ISO_OP_ALLGATHER, alg)
    pinfo = iso.iso_plan_info(plan)
    rounds = _plan_rounds(plan)
    send = RNG.integers(0, 256, size=(p, m), dtype=np.uint8)
    recv, written = _replay(dims, offsets, iso.ISO_OP_ALLGATHER, rounds, pinfo["work_slots"], send, m)
    assert np.array_equal(recv, orc.allgather(dims, offsets, send))
    assert {(iso.ISO_BUF_RECV, i) for i in range(s)} <= written
    if alg in (iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_BYDIM):
        order = pinfo["dim_order"][:len(dims)]
        assert sorted(order) == list(range(len(dims)))
        can = orc.canonical(dims, offsets)
        n_self = sum(1 for C in can if not any(C))
        dup_extra = sum(can[:i].count(C) > 0 and any(C) for i, C in enumerate(can))
        assert pinfo["entries"] == orc.direct_allgather_volume(dims, offsets, order) + dup_extra + n_self
        assert pinfo["entries"] - n_self == iso.iso_neighborhood_info(comm)["allgather_moves"]
        if alg == iso.ISO_ALG_COMBINED:
            n_shift = sum(1 for r in rounds if r[0]["kind"] == iso.ISO_ROUND_SHIFT)
            assert n_shift == len(orc.direct_rounds(dims, offsets))
    elif alg == iso.ISO_ALG_COMBINED_STAGED:
        # the trie's moves, plus one copy for every block that had to be complete before the last launch
        n_self = sum(1 for C in orc.canonical(dims, offsets) if not any(C))
        moves = iso.iso_neighborhood_info(comm)["allgather_moves"]
        copies = sum(1 for e in rounds[-1][1] if e["dim"] < 0) - n_self if s else 0
        assert 0 <= copies <= s and pinfo["entries"] == moves + n_self + copies
        _check_staged_shape(iso.ISO_OP_ALLGATHER, dims, offsets, rounds)
    elif alg == iso.ISO_ALG_ONEHOP:
        # Proposition 2: the same D steps, W block-moves (plus one per repeated offset)
        order = pinfo["dim_order"][:len(dims)]
        raw = [tuple(C) for C in offsets]
        raw_self = sum(1 for C in raw if not any(C))
        dup_extra = sum(raw[:i].count(C) > 0 and any(C) for i, C in enumerate(raw))
        n_shift = sum(1 for r in rounds if r[0]["kind"] == iso.ISO_ROUND_SHIFT)
        assert n_shift == orc.onehop_rounds(offsets)
        assert pinfo["entries"] == orc.onehop_allgather_volume(offsets, order) + dup_extra + raw_self
        assert pinfo["entries"] - raw_self - dup_extra <= orc.onehop_alltoall_volume(offsets)


def test_figure1_example_plan(golden):
    offs = [tuple(int(x) for x in t.split(",")) for t in golden["fig1_offsets"].split(";")]
    comm = iso.iso_neighborhood_create((16, 16, 16), offs)
    info = iso.iso_neighborhood_info(comm)
    assert info["rounds"] == int(golden["fig1_direct_rounds"])
    assert info["alltoall_moves"] == int(golden["fig1_direct_V"])
    assert info["allgather_moves"] == int(golden["fig1_direct_W"])
    assert info["self_slots"] == 1
    ag = iso.iso_plan_create(comm, iso.ISO_OP_ALLGATHER)
    pi = iso.iso_plan_info(ag)
    assert pi["dim_order"][:3] == [0, 1, 2]
    shift = [(i, e) for i, e in _plan_rounds(ag) if i["kind"] == iso.ISO_ROUND_SHIFT]
    assert [i["n_entries"] for i, _ in shift] == [int(x) for x in golden["fig1_direct_allgather_k"].split(",")]
    # four trie nodes are not neighbours themselves: (3), (4), (3,3), (4,1); those of the
    # first level are still being read when the second level is written: four slots
    temps = [e for _, es in shift for e in es if e["dst_buf"] == iso.ISO_BUF_WORK]
    assert len(temps) == 4 and pi["work_slots"] == 4
    a2a = iso.iso_plan_create(comm, iso.ISO_OP_ALLTOALL)
    shift = [i for i, _ in _plan_rounds(a2a) if i["kind"] == iso.ISO_ROUND_SHIFT]
    assert [i["n_entries"] for i in shift] == [int(x) for x in golden["fig1_direct_alltoall_k"].split(",")]


def test_config_constants():
    want = {  # name prefix -> (rounds, a2a moves, allgather moves, a2a k per round)
        "c1": (4, 12, 8), "c2": (6, 54, 26), "c3": (8, 16, 12), "c4": (6, 54, 26),
    }
    for cfg in gen.CONFIGS:
        comm = iso.iso_neighborhood_create(cfg.dims, cfg.offsets)
        info = iso.iso_neighborhood_info(comm)
        key = cfg.name[:2]
        if key in want:
            assert (info["rounds"], info["alltoall_moves"], info["allgather_moves"]) == want[key]
        else:
            assert info["rounds"] == len(orc.direct_rounds(cfg.dims, cfg.offsets)) <= 30
            assert info["allgather_moves"] <= info["alltoall_moves"]
    c2 = gen.get_config(2)
    comm = iso.iso_neighborhood_create(c2.dims, c2.offsets)
    a2a = [i["n_entries"] for i, _ in _plan_rounds(iso.iso_plan_create(comm, iso.ISO_OP_ALLTOALL))]
    ag = [i["n_entries"] for i, _ in _plan_rounds(iso.iso_plan_create(comm, iso.ISO_OP_ALLGATHER))]
    assert a2a == [9] * 6 and sorted(ag) == [1, 1, 3, 3, 9, 9]
    assert iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLGATHER, iso.ISO_ALG_COMBINED, 256) == 0
    assert iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, 256) == 20 * 32768 * 256
    assert iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_SX_FUSED, 256) == 0


def test_allgather_workspace_slots_are_reused():
    cfg = gen.get_config(5)
    comm = iso.iso_neighborhood_create(cfg.dims, cfg.offsets)
    plan = iso.iso_plan_create(comm, iso.ISO_OP_ALLGATHER)
    pi = iso.iso_plan_info(plan)
    temps = sum(1 for _, es in _plan_rounds(plan) for e in es if e["dst_buf"] == iso.ISO_BUF_WORK)
    assert 0 < pi["work_slots"] < temps


FASTDIV_TEST = r"""
#include <cstdio>
#include <cstdint>
#include "iso_fastdiv.hpp"
int main() {
    const uint32_t divs[] = {1,2,3,5,7,8,9,16,26,27,31,32,33,63,64,255,256,257,1000,4095,4096,
                             65535,65536,65537,262144,1000003,(1u<<30)-1,1u<<30,(1u<<31)-1,1u<<31};
    uint64_t x = 88172645463325252ull; long bad = 0, n = 0;
    for (uint32_t d : divs) {
        iso::FastDiv f = iso::make_fastdiv(d);
        const uint32_t edge[] = {0,1,d-1,d,d+1,2*d-1,2*d,0xFFFFFFFFu,0xFFFFFFFEu,0x80000000u,0x7FFFFFFFu};
        for (uint32_t v : edge) { uint32_t q,r; iso::fast_divmod(v,f,q,r); bad += (q!=v/d)||(r!=v%d); ++n; }
        for (int i = 0; i < 200000; ++i) {
            x ^= x << 13; x ^= x >> 7; x ^= x << 17;
            uint32_t v = (uint32_t)x; uint32_t q,r; iso::fast_divmod(v,f,q,r);
            bad += (q!=v/d)||(r!=v%d); ++n;
        }
    }
    std::printf("%ld %ld\n", n, bad);
    return bad != 0;
}
"""


def test_fastdiv_is_exact_on_the_host():
    with tempfile.TemporaryDirectory() as td:
        src = os.path.join(td, "t.cpp")
        open(src, "w").write(FASTDIV_TEST)
        exe = os.path.join(td, "t")
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-I",
                               os.path.join(ROOT, "paper_1606_07676_amd", "csrc"), src, "-o", exe])
        out = subprocess.check_output([exe], text=True).split()
        assert int(out[0]) > 1_000_000 and int(out[1]) == 0


def test_schedule_builder_under_address_and_ub_sanitizers():
    """The host-side schedule builder (pure C++) compiled with -fsanitize=address,undefined
    and driven with seeded random tori, meshes and neighbourhoods through every algorithm."""
    csrc = os.path.join(ROOT, "paper_1606_07676_amd", "csrc")
    with tempfile.TemporaryDirectory() as td:
        exe = os.path.join(td, "plan_san")
        subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
                               "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-I", csrc, "-I", os.path.join(ROOT, "include"),
                               os.path.join(ROOT, "tests", "plan_sanitizer_driver.cpp"),
                               os.path.join(csrc, "iso_plan.cpp"), "-o", exe])
        # the sanitizer runtimes are linked statically: a preloaded library may then come first
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
        out = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
        assert out.returncode == 0, out.stderr[-2000:]
        assert int(out.stdout.split()[0]) > 3000


# ---------------------------------------------------------------- meshes (non-periodic dimensions)

MESHES = [
    ((5,), (0,), [(1,), (-2,), (7,), (0,)]),
    ((4, 3), (0, 0), gen.moore(2, 1)),
    ((4, 3), (1, 0), gen.moore(2, 1) + [(0, 0), (5, 1), (1, 1)]),
    ((3, 4, 2), (0, 1, 0), gen.moore(3, 1)),
    ((6, 5), (0, 0), gen.von_neumann(2, 2)),
    ((5, 4, 3), (0, 0, 0), gen.moore(3, 1)),
    ((4, 4, 4), (0, 0, 1), [(0, 0, 0), (0, 0, 1), (1, 0, 0), (1, 1, 0), (1, 1, 1), (3, 2, 0), (3, 3, 2),
                            (2, 0, 1), (2, 0, 2), (-1, 1, 1)]),
]
MESH_ALGS = [iso.ISO_ALG_COMBINED, iso.ISO_ALG_COMBINED_BYDIM, iso.ISO_ALG_SX_ROUNDS, iso.ISO_ALG_SX_FUSED]


def _replay_mesh(dims, periodic, offsets, op, order, rounds, work_slots, send, m):
    """Plan replay on a mesh: an entry's move happens at rank R only if R - C^ref is
    inside the mesh in the non-periodic dimensions routed so far."""
    d, s = len(dims), len(offsets)
    p = int(np.prod(dims))
    shape = tuple(dims)
    eff = [tuple(c % n if per else c for c, n, per in zip(C, dims, periodic)) for C in offsets]
    grid = np.indices(shape)
    bufs = {
        iso.ISO_BUF_SEND: send.reshape(shape + ((s, m) if op == iso.ISO_OP_ALLTOALL else (1, m))),
        iso.ISO_BUF_RECV: np.full(shape + (max(s, 1), m), 0xEE, np.uint8),
        iso.ISO_BUF_WORK: np.full(shape + (max(work_slots, 1), m), 0xDD, np.uint8),
    }
    for info, entries in rounds:
        if info["kind"] == iso.ISO_ROUND_SHIFT:
            routed = order[:order.index(info["dim"]) + 1]
        elif info["kind"] == iso.ISO_ROUND_VECTOR:
            routed = list(range(d))
        else:
            routed = []
        reads, writes, staged = set(), set(), []
        for e in entries:
            src = bufs[e["src_buf"]][..., e["src_slot"], :]
            C = eff[e["ref"]]
            valid = np.ones(shape, bool)
            for l in routed:
                if not periodic[l] and C[l] != 0:
                    t = grid[l] - C[l]
                    valid &= (t >= 0) & (t < dims[l])
            if info["kind"] == iso.ISO_ROUND_SHIFT:
                assert e["shift"] == C[info["dim"]]
                data = np.roll(src, e["shift"], axis=info["dim"])
            elif info["kind"] == iso.ISO_ROUND_SELF:
                data = src.copy()
            else:
                data = np.roll(src, eff[e["neighbor"]], axis=tuple(range(d)))
            staged.append((e, data, valid))
            reads.add((e["src_buf"], e["src_slot"]))
            assert (e["dst_buf"], e["dst_slot"]) not in writes
            writes.add((e["dst_buf"], e["dst_slot"]))
            assert e["dst_buf"] != iso.ISO_BUF_SEND
        assert not (reads & writes)
        for e, data, valid in staged:
            bufs[e["dst_buf"]][..., e["dst_slot"], :][valid] = data[valid]
    return bufs[iso.ISO_BUF_RECV].reshape(p, max(s, 1), m)[:, :s]


@pytest.mark.parametrize("alg", MESH_ALGS)
@pytest.mark.parametrize("dims,periodic,offsets", MESHES)
def test_mesh_plans_reach_the_oracle_result(dims, periodic, offsets, alg):
    p, s, m = int(np.prod(dims)), len(offsets), 2
    comm = iso.iso_neighborhood_create_mesh(dims, periodic, offsets)
    for op in (iso.ISO_OP_ALLTOALL, iso.ISO_OP_ALLGATHER):
        plan = iso.iso_plan_create(comm, op, alg)
        pinfo = iso.iso_plan_info(plan)
        rounds = _plan_rounds(plan)
        order = pinfo["dim_order"][:len(dims)]
        if op == iso.ISO_OP_ALLTOALL:
            send = RNG.integers(0, 256, size=(p, s, m), dtype=np.uint8)
            want = orc.alltoall_mesh(dims, periodic, offsets, send, np.full((p, s, m), 0xEE, np.uint8))
            # a block in transit never sits in the receive buffer of a mesh
            for info, entries in rounds:
                for e in entries:
                    assert not (e["src_buf"] == iso.ISO_BUF_RECV)
        else:
            send = RNG.integers(0, 256, size=(p, m), dtype=np.uint8)
            want = orc.allgather_mesh(dims, periodic, offsets, send, np.full((p, s, m), 0xEE, np.uint8))
        got = _replay_mesh(dims, periodic, offsets, op, order, rounds, pinfo["work_slots"], send, m)
        assert np.array_equal(got, want), (dims, periodic, alg, op)


def test_onehop_is_refused_on_a_mesh_and_full_periodicity_is_the_torus():
    comm = iso.iso_neighborhood_create_mesh((4, 4), (1, 0), gen.moore(2, 1))
    with pytest.raises(iso.IsoError) as e:
        iso.iso_plan_create(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_ONEHOP)
    assert e.value.status == iso.ISO_ERR_ARG
    a = iso.iso_neighborhood_create_mesh((4, 4), (1, 1), gen.moore(2, 1))
    b = iso.iso_neighborhood_create((4, 4), gen.moore(2, 1))
    pa, pb = iso.iso_plan_create(a, iso.ISO_OP_ALLTOALL), iso.iso_plan_create(b, iso.ISO_OP_ALLTOALL)
    assert _plan_rounds(pa) == _plan_rounds(pb)


# ---------------------------------------------------------------- seeded random sweep

def _random_case(rng, mesh, d=None):
    if d is None:
        d = int(rng.integers(1, 5))
        dims = tuple(int(x) for x in rng.integers(1, 6, size=d))
    else:                       # many dimensions, few ranks
        while True:
            dims = tuple(int(x) for x in rng.choice([1, 2, 2, 3], size=d))
            if int(np.prod(dims)) <= 1024:
                break
    s = int(rng.integers(0, 13))
    span = int(rng.integers(1, 8))
    offsets = [tuple(int(x) for x in rng.integers(-span, span + 1, size=d)) for _ in range(s)]
    for _ in range(int(rng.integers(0, 3))):                       # repeats and the zero vector
        if offsets:
            offsets.append(offsets[int(rng.integers(0, len(offsets)))])
    if rng.integers(0, 3) == 0:
        offsets.append((0,) * d)
    periodic = tuple(int(x) for x in rng.integers(0, 2, size=d)) if mesh else (1,) * d
    return dims, periodic, offsets


@pytest.mark.parametrize("seed", range(48))
def test_random_torus_plans_reach_the_oracle_result(seed):
    """Random tori (sizes 1..5, so offsets alias and wrap several times), random signed
    offsets with repeats and zero vectors: every algorithm's plan, replayed on the host,
    gives the definition, without hazards.  Seeds from 40 on: 7 to 16 dimensions."""
    rng = np.random.default_rng(1000 + seed)
    dims, _, offsets = _random_case(rng, mesh=False, d=None if seed < 40 else (7, 8, 9, 10, 12, 14, 16, 16)[seed - 40])
    p, s, m = int(np.prod(dims)), len(offsets), 2
    comm = iso.iso_neighborhood_create(dims, np.asarray(offsets, np.int32).reshape(s, len(dims)))
    a2a = rng.integers(0, 256, size=(p, s, m), dtype=np.uint8)
    ag = rng.integers(0, 256, size=(p, m), dtype=np.uint8)
    want_a2a, want_ag = orc.alltoall(dims, offsets, a2a), orc.allgather(dims, offsets, ag)
    for alg in ALGS:
        for op, send, want in ((iso.ISO_OP_ALLTOALL, a2a, want_a2a), (iso.ISO_OP_ALLGATHER, ag, want_ag)):
            plan = iso.iso_plan_create(comm, op, alg)
            pinfo = iso.iso_plan_info(plan)
            recv, written = _replay(dims, offsets, op, _plan_rounds(plan), pinfo["work_slots"], send, m)
            assert np.array_equal(recv, want), (dims, offsets, alg, op)
            assert {(iso.ISO_BUF_RECV, i) for i in range(s)} <= written


@pytest.mark.parametrize("seed", range(36))
def test_random_mesh_plans_reach_the_oracle_result(seed):
    rng = np.random.default_rng(2000 + seed)
    dims, periodic, offsets = _random_case(rng, mesh=True, d=None if seed < 30 else (7, 8, 10, 12, 16, 16)[seed - 30])
    p, s, m = int(np.prod(dims)), len(offsets), 2
    comm = iso.iso_neighborhood_create_mesh(dims, periodic, np.asarray(offsets, np.int32).reshape(s, len(dims)))
    a2a = rng.integers(0, 256, size=(p, s, m), dtype=np.uint8)
    ag = rng.integers(0, 256, size=(p, m), dtype=np.uint8)
    keep = np.full((p, s, m), 0xEE, np.uint8)
    want_a2a = orc.alltoall_mesh(dims, periodic, offsets, a2a, keep.copy())
    want_ag = orc.allgather_mesh(dims, periodic, offsets, ag, keep.copy())
    for alg in MESH_ALGS:
        for op, send, want in ((iso.ISO_OP_ALLTOALL, a2a, want_a2a), (iso.ISO_OP_ALLGATHER, ag, want_ag)):
            plan = iso.iso_plan_create(comm, op, alg)
            pinfo = iso.iso_plan_info(plan)
            order = pinfo["dim_order"][:len(dims)]
            got = _replay_mesh(dims, periodic, offsets, op, order, _plan_rounds(plan), pinfo["work_slots"],
                               send, m)
            assert np.array_equal(got, want), (dims, periodic, offsets, alg, op)


def test_workspace_names_of_the_message_combining_schedule():
    comm = iso.iso_neighborhood_create((9, 9, 9), gen.positive_octant(3, 3))
    for m in (0, 1, 48, 4096):
        assert iso.iso_alltoall_workspace_bytes(comm, m) == \
            iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, m)
        assert iso.iso_allgather_workspace_bytes(comm, m) == \
            iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLGATHER, iso.ISO_ALG_COMBINED, m)
    assert iso.iso_alltoall_workspace_bytes(comm, 16) > 0
    fig1 = iso.iso_neighborhood_create((9, 9, 9), [(0, 0, 0), (0, 0, 1), (1, 0, 0), (1, 1, 0), (1, 1, 1), (3, 2, 0),
                                                    (3, 3, 2), (4, 0, 1), (4, 0, 2), (4, 1, 1)])
    assert iso.iso_allgather_workspace_bytes(fig1, 16) == 4 * 729 * 16       # Figure 1: four stored nodes are no neighbours
    # irregular allgather: every process sends one size, as the init call demands
    s = len(gen.positive_octant(3, 3))
    assert iso.iso_workspace_bytes_v(comm, iso.ISO_OP_ALLGATHER, iso.ISO_ALG_COMBINED, [24] * s) == \
        iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLGATHER, iso.ISO_ALG_COMBINED, 24)
    with pytest.raises(iso.IsoError) as e:
        iso.iso_workspace_bytes_v(comm, iso.ISO_OP_ALLGATHER, iso.ISO_ALG_COMBINED, [24] * (s - 1) + [25])
    assert e.value.status == iso.ISO_ERR_ARG
    iso.iso_workspace_bytes_v(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, [24] * (s - 1) + [25])


def test_sizes_that_would_overflow_are_refused():
    comm = iso.iso_neighborhood_create((32, 32, 32), gen.moore(3, 1))
    for alg in ALGS:
        with pytest.raises(iso.IsoError) as e:
            iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, alg, 1 << 62)
        assert e.value.status == iso.ISO_ERR_TOO_LARGE
        with pytest.raises(iso.IsoError) as e:
            iso.iso_workspace_bytes_v(comm, iso.ISO_OP_ALLGATHER, alg, [1 << 61] * 26)
        assert e.value.status == iso.ISO_ERR_TOO_LARGE
    assert iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, 256) == 20 * 32768 * 256
    # the one-hop schedule needs one launch per unit of coordinate: absurd counts are refused
    far = iso.iso_neighborhood_create((5, 5), [(70000, 0), (0, -1)])
    with pytest.raises(iso.IsoError) as e:
        iso.iso_plan_create(far, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_ONEHOP)
    assert e.value.status == iso.ISO_ERR_TOO_LARGE
    assert iso.iso_plan_info(iso.iso_plan_create(far, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED))["launches"] == 2   # a same-rank copy (70000 = 0 mod 5) and one shift


def test_header_is_plain_c(tmp_path):
    """include/iso.h is the boundary of a C ABI: a C99 compiler must take it as it is, pedantically."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if not gcc:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_iso_h.c"
    src.write_text('#include "iso.h"\n'
                   "int main(void) { iso_plan_entry_t e; iso_comm_info_t c; e.dim = ISO_ROUND_DELIVER; c.d = e.dim;\n"
                   "  return c.d == ISO_ALG_COMBINED_STAGED ? 1 : 0; }\n")
    out = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                          "-c", str(src), "-o", str(tmp_path / "use_iso_h.o")],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert out.returncode == 0, out.stdout
