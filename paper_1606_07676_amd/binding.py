"""ctypes binding of libiso.so: same names as include/iso.h, argument marshalling
only.  A missing library is an error (there is no fallback path): build it with
`python -m paper_1606_07676_amd.build` or `__graft_entry__.build()`."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libiso.so")
_lib = None

ISO_MAX_DIMS = 16
(ISO_SUCCESS, ISO_ERR_ARG, ISO_ERR_OVERLAP, ISO_ERR_WORKSPACE, ISO_ERR_HIP, ISO_ERR_NOMEM,
 ISO_ERR_TOO_LARGE, ISO_ERR_POINTER, ISO_ERR_SCRATCH) = range(9)
ISO_NOALLOC_SCRATCH_BYTES, ISO_NOALLOC_TABLE_BYTES = 32 << 20, 256 << 10
ISO_OP_ALLTOALL, ISO_OP_ALLGATHER = 0, 1
ISO_ALG_COMBINED, ISO_ALG_COMBINED_BYDIM, ISO_ALG_SX_ROUNDS, ISO_ALG_SX_FUSED, ISO_ALG_ONEHOP = 0, 1, 2, 3, 4
ISO_ALG_COMBINED_STAGED = 5
ISO_BUF_SEND, ISO_BUF_RECV, ISO_BUF_WORK = 0, 1, 2
ISO_LAYOUT_RANK_MAJOR, ISO_LAYOUT_SLOT_MAJOR = 0, 1
ISO_SX_LAUNCHES, ISO_SX_FUSED = 0, 1
ISO_GRAPH_OFF, ISO_GRAPH_CHAIN, ISO_GRAPH_BRANCHES = 0, 1, 2
ISO_ROUND_SHIFT, ISO_ROUND_SELF, ISO_ROUND_VECTOR, ISO_ROUND_DELIVER = 0, 1, 2, 3


class IsoError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = f"{where}: status {status}"
        try:
            msg += f" ({iso_error_string(status)})"
            if status == ISO_ERR_HIP:
                msg += f", hipError_t {iso_last_hip_error()}"
        except Exception:
            pass
        super().__init__(msg)


class iso_comm_info_t(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("s", ctypes.c_int32), ("p", ctypes.c_int64),
                ("rounds", ctypes.c_int32), ("self_slots", ctypes.c_int32),
                ("alltoall_moves", ctypes.c_int64), ("allgather_moves", ctypes.c_int64)]


class iso_plan_info_t(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int32), ("algorithm", ctypes.c_int32),
                ("launches", ctypes.c_int32), ("work_slots", ctypes.c_int32),
                ("entries", ctypes.c_int64), ("dim_order", ctypes.c_int32 * ISO_MAX_DIMS)]


class iso_round_info_t(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("dim", ctypes.c_int32),
                ("n_entries", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class iso_plan_entry_t(ctypes.Structure):
    _fields_ = [("src_buf", ctypes.c_int32), ("src_slot", ctypes.c_int32),
                ("dst_buf", ctypes.c_int32), ("dst_slot", ctypes.c_int32),
                ("shift", ctypes.c_int32), ("neighbor", ctypes.c_int32),
                ("ref", ctypes.c_int32), ("dim", ctypes.c_int32)]


class iso_request_info_t(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int32), ("algorithm", ctypes.c_int32),
                ("launches", ctypes.c_int32), ("vector_bytes", ctypes.c_int32),
                ("p", ctypes.c_int64), ("s", ctypes.c_int64),
                ("block_bytes", ctypes.c_uint64), ("entries", ctypes.c_int64),
                ("bytes_read", ctypes.c_uint64), ("bytes_written", ctypes.c_uint64),
                ("delivered_bytes", ctypes.c_uint64), ("workspace_bytes", ctypes.c_uint64)]


def _struct_dict(st):
    out = {}
    for name, _ in st._fields_:
        v = getattr(st, name)
        out[name] = list(v) if hasattr(v, "__len__") else v
    return out


def library_path():
    return _LIB_PATH


_VP, _I, _SZ = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
_PROTOTYPES = {
    "iso_neighborhood_create": ([_I, _VP, _I, _VP, ctypes.POINTER(_VP)], _I),
    "iso_neighborhood_create_mesh": ([_I, _VP, _VP, _I, _VP, ctypes.POINTER(_VP)], _I),
    "iso_neighborhood_info": ([_VP, ctypes.POINTER(iso_comm_info_t)], _I),
    "iso_neighborhood_free": ([ctypes.POINTER(_VP)], _I),
    "iso_plan_create": ([_VP, _I, _I, ctypes.POINTER(_VP)], _I),
    "iso_plan_info": ([_VP, ctypes.POINTER(iso_plan_info_t)], _I),
    "iso_plan_round": ([_VP, _I, ctypes.POINTER(iso_round_info_t)], _I),
    "iso_plan_entries": ([_VP, _I, ctypes.POINTER(iso_plan_entry_t), _I], _I),
    "iso_plan_free": ([ctypes.POINTER(_VP)], _I),
    "iso_workspace_bytes": ([_VP, _I, _I, _SZ, ctypes.POINTER(_SZ)], _I),
    "iso_alltoall_workspace_bytes": ([_VP, _SZ, ctypes.POINTER(_SZ)], _I),
    "iso_allgather_workspace_bytes": ([_VP, _SZ, ctypes.POINTER(_SZ)], _I),
    "iso_neighbor_alltoall_sx_init": ([_VP, _VP, _SZ, _I, _VP, ctypes.POINTER(_VP)], _I),
    "iso_neighbor_allgather_sx_init": ([_VP, _VP, _SZ, _I, _VP, ctypes.POINTER(_VP)], _I),
    "iso_neighbor_alltoall_init": ([_VP, _VP, _SZ, _VP, _SZ, _VP, _I, ctypes.POINTER(_VP)], _I),
    "iso_neighbor_allgather_init": ([_VP, _VP, _SZ, _VP, _SZ, _VP, _I, ctypes.POINTER(_VP)], _I),
    "iso_neighbor_alltoall_init_layout": ([_VP, _VP, _SZ, _I, _VP, _SZ, _VP, _I, ctypes.POINTER(_VP)], _I),
    "iso_neighbor_allgather_init_layout": ([_VP, _VP, _SZ, _I, _VP, _SZ, _VP, _I, ctypes.POINTER(_VP)], _I),
    "iso_workspace_bytes_v": ([_VP, _I, _I, _VP, ctypes.POINTER(_SZ)], _I),
    "iso_neighbor_alltoallv_init": ([_VP, _VP, _VP, _SZ, _VP, _VP, _VP, _SZ, _VP, _SZ, _VP, _I,
                                     ctypes.POINTER(_VP)], _I),
    "iso_neighbor_allgatherv_init": ([_VP, _SZ, _SZ, _VP, _VP, _VP, _SZ, _VP, _SZ, _VP, _I,
                                      ctypes.POINTER(_VP)], _I),
    "iso_neighbor_alltoallv_init_layout": ([_VP, _VP, _VP, _SZ, _VP, _VP, _VP, _SZ, _I, _VP, _SZ, _VP, _I,
                                            ctypes.POINTER(_VP)], _I),
    "iso_neighbor_allgatherv_init_layout": ([_VP, _SZ, _SZ, _VP, _VP, _VP, _SZ, _I, _VP, _SZ, _VP, _I,
                                             ctypes.POINTER(_VP)], _I),
    "iso_neighbor_alltoallw_init": ([_VP, _VP, _VP, _SZ, _VP, _VP, _VP, _SZ, _VP, _SZ, _VP, _I,
                                     ctypes.POINTER(_VP)], _I),
    "iso_neighbor_allgatherw_init": ([_VP, _SZ, _SZ, _VP, _VP, _VP, _SZ, _VP, _SZ, _VP, _I,
                                      ctypes.POINTER(_VP)], _I),
    "iso_neighbor_alltoall_noalloc": ([_VP, _VP, _SZ, _VP, _I, _VP], _I),
    "iso_start": ([_VP, _VP], _I),
    "iso_start_range": ([_VP, _I, _I, _VP], _I),
    "iso_request_set_graph": ([_VP, _I], _I),
    "iso_wait": ([_VP], _I),
    "iso_request_info": ([_VP, ctypes.POINTER(iso_request_info_t)], _I),
    "iso_request_plan": ([_VP, ctypes.POINTER(_VP)], _I),
    "iso_request_free": ([ctypes.POINTER(_VP)], _I),
    "iso_error_string": ([_I], ctypes.c_char_p),
    "iso_last_hip_error": ([], _I),
    "iso_copy_reference": ([_VP, _VP, _SZ, _VP], _I),
}


def load_library():
    """dlopen libiso.so and set the prototypes; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build the HIP library first "
                "(python -m paper_1606_07676_amd.build); there is no fallback path")
        # PyTorch ships its own HIP runtime under the same soname as the system's.
        # Loading it first makes the dynamic linker bind libiso to that one copy, so
        # that torch's device pointers and streams are valid handles in libiso.
        import torch  # noqa: F401
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (argtypes, restype) in _PROTOTYPES.items():
            fn = getattr(lib, name)
            fn.argtypes = argtypes
            fn.restype = restype
        _lib = lib
    return _lib


def _check(status, where):
    if status != ISO_SUCCESS:
        raise IsoError(status, where)


def _ptr(x):
    """Device address of a torch tensor (must be contiguous), an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x or None
    if hasattr(x, "data_ptr"):
        if not x.is_contiguous():
            raise ValueError("buffers must be contiguous")
        return x.data_ptr() or None
    raise TypeError("expected a torch tensor, an integer address or None")


def _nbytes(x, given):
    if given is not None:
        return int(given)
    if x is None:
        return 0
    if hasattr(x, "numel"):
        return x.numel() * x.element_size()
    raise TypeError("workspace_bytes is required with a raw address")


def _stream_handle(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


class _Handle:
    _free_name = None

    def __init__(self, handle, owned=True):
        self._h = ctypes.c_void_p(handle)
        self._owned = owned

    @property
    def handle(self):
        if not self._h:
            raise ValueError("handle already freed")
        return self._h

    def free(self):
        if self._h and self._owned:
            getattr(load_library(), self._free_name)(ctypes.byref(self._h))
        self._h = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class Comm(_Handle):
    _free_name = "iso_neighborhood_free"


class Plan(_Handle):
    _free_name = "iso_plan_free"


class Request(_Handle):
    _free_name = "iso_request_free"

    def __init__(self, handle, keepalive):
        super().__init__(handle)
        self._keepalive = keepalive      # tensors bound to the request


# ---- functions, named as in iso.h ------------------------------------------

def iso_neighborhood_create(dims, rel_coords):
    """dims: d ints; rel_coords: s vectors of d ints (or a flat list)."""
    dims_a = np.ascontiguousarray(dims, dtype=np.int32).reshape(-1)
    d = dims_a.size
    rel = np.ascontiguousarray(rel_coords, dtype=np.int32).reshape(-1)
    if d == 0 or rel.size % max(d, 1):
        raise ValueError("rel_coords must hold s*d integers")
    h = ctypes.c_void_p()
    st = load_library().iso_neighborhood_create(d, dims_a.ctypes.data, rel.size // d,
                                                rel.ctypes.data if rel.size else None,
                                                ctypes.byref(h))
    _check(st, "iso_neighborhood_create")
    return Comm(h.value)


def iso_neighborhood_create_mesh(dims, periodic, rel_coords):
    """As iso_neighborhood_create; periodic: d flags (False = that dimension does not wrap)."""
    dims_a = np.ascontiguousarray(dims, dtype=np.int32).reshape(-1)
    d = dims_a.size
    per = np.ascontiguousarray([1 if x else 0 for x in periodic], dtype=np.int32)
    rel = np.ascontiguousarray(rel_coords, dtype=np.int32).reshape(-1)
    if d == 0 or per.size != d or rel.size % d:
        raise ValueError("need d periodic flags and s*d relative coordinates")
    h = ctypes.c_void_p()
    st = load_library().iso_neighborhood_create_mesh(d, dims_a.ctypes.data, per.ctypes.data, rel.size // d,
                                                     rel.ctypes.data if rel.size else None, ctypes.byref(h))
    _check(st, "iso_neighborhood_create_mesh")
    return Comm(h.value)


def iso_neighborhood_info(comm):
    info = iso_comm_info_t()
    _check(load_library().iso_neighborhood_info(comm.handle, ctypes.byref(info)), "iso_neighborhood_info")
    return _struct_dict(info)


def iso_neighborhood_free(comm):
    comm.free()


def iso_plan_create(comm, op, algorithm=ISO_ALG_COMBINED):
    h = ctypes.c_void_p()
    _check(load_library().iso_plan_create(comm.handle, op, algorithm, ctypes.byref(h)), "iso_plan_create")
    return Plan(h.value)


def iso_plan_info(plan):
    info = iso_plan_info_t()
    _check(load_library().iso_plan_info(plan.handle, ctypes.byref(info)), "iso_plan_info")
    return _struct_dict(info)


def iso_plan_round(plan, r):
    info = iso_round_info_t()
    _check(load_library().iso_plan_round(plan.handle, r, ctypes.byref(info)), "iso_plan_round")
    return _struct_dict(info)


def iso_plan_entries(plan, r):
    n = iso_plan_round(plan, r)["n_entries"]
    arr = (iso_plan_entry_t * max(n, 1))()
    _check(load_library().iso_plan_entries(plan.handle, r, arr, n), "iso_plan_entries")
    return [_struct_dict(arr[i]) for i in range(n)]


def iso_plan_free(plan):
    plan.free()


def iso_workspace_bytes(comm, op, algorithm, m):
    out = ctypes.c_size_t()
    _check(load_library().iso_workspace_bytes(comm.handle, op, algorithm, m, ctypes.byref(out)),
           "iso_workspace_bytes")
    return out.value


def iso_alltoall_workspace_bytes(comm, m):
    out = ctypes.c_size_t()
    _check(load_library().iso_alltoall_workspace_bytes(comm.handle, m, ctypes.byref(out)),
           "iso_alltoall_workspace_bytes")
    return out.value


def iso_allgather_workspace_bytes(comm, m):
    out = ctypes.c_size_t()
    _check(load_library().iso_allgather_workspace_bytes(comm.handle, m, ctypes.byref(out)),
           "iso_allgather_workspace_bytes")
    return out.value


def _sx_init(name, sendbuf, recvbuf, m, mode, comm):
    h = ctypes.c_void_p()
    st = getattr(load_library(), name)(_ptr(sendbuf), _ptr(recvbuf), m, mode, comm.handle, ctypes.byref(h))
    _check(st, name)
    return Request(h.value, (sendbuf, recvbuf))


def iso_neighbor_alltoall_sx_init(sendbuf, recvbuf, m, mode, comm):
    return _sx_init("iso_neighbor_alltoall_sx_init", sendbuf, recvbuf, m, mode, comm)


def iso_neighbor_allgather_sx_init(sendbuf, recvbuf, m, mode, comm):
    return _sx_init("iso_neighbor_allgather_sx_init", sendbuf, recvbuf, m, mode, comm)


def _init(name, sendbuf, recvbuf, m, workspace, workspace_bytes, comm, algorithm):
    h = ctypes.c_void_p()
    fn = getattr(load_library(), name)
    st = fn(_ptr(sendbuf), _ptr(recvbuf), m, _ptr(workspace), _nbytes(workspace, workspace_bytes),
            comm.handle, algorithm, ctypes.byref(h))
    _check(st, name)
    return Request(h.value, (sendbuf, recvbuf, workspace))


def iso_neighbor_alltoall_init(sendbuf, recvbuf, m, workspace, comm,
                               algorithm=ISO_ALG_COMBINED, workspace_bytes=None):
    return _init("iso_neighbor_alltoall_init", sendbuf, recvbuf, m, workspace, workspace_bytes,
                 comm, algorithm)


def iso_neighbor_allgather_init(sendbuf, recvbuf, m, workspace, comm,
                                algorithm=ISO_ALG_COMBINED, workspace_bytes=None):
    return _init("iso_neighbor_allgather_init", sendbuf, recvbuf, m, workspace, workspace_bytes,
                 comm, algorithm)


def _init_layout(name, sendbuf, recvbuf, m, layout, workspace, workspace_bytes, comm, algorithm):
    h = ctypes.c_void_p()
    fn = getattr(load_library(), name)
    st = fn(_ptr(sendbuf), _ptr(recvbuf), m, layout, _ptr(workspace), _nbytes(workspace, workspace_bytes),
            comm.handle, algorithm, ctypes.byref(h))
    _check(st, name)
    return Request(h.value, (sendbuf, recvbuf, workspace))


def iso_neighbor_alltoall_init_layout(sendbuf, recvbuf, m, layout, workspace, comm,
                                      algorithm=ISO_ALG_COMBINED, workspace_bytes=None):
    return _init_layout("iso_neighbor_alltoall_init_layout", sendbuf, recvbuf, m, layout, workspace,
                        workspace_bytes, comm, algorithm)


def iso_neighbor_allgather_init_layout(sendbuf, recvbuf, m, layout, workspace, comm,
                                       algorithm=ISO_ALG_COMBINED, workspace_bytes=None):
    return _init_layout("iso_neighbor_allgather_init_layout", sendbuf, recvbuf, m, layout, workspace,
                        workspace_bytes, comm, algorithm)


def _size_array(values):
    return np.ascontiguousarray(values, dtype=np.uintp).reshape(-1)


def iso_workspace_bytes_v(comm, op, algorithm, sizes):
    out = ctypes.c_size_t()
    arr = _size_array(sizes)
    _check(load_library().iso_workspace_bytes_v(comm.handle, op, algorithm,
                                                arr.ctypes.data if arr.size else None, ctypes.byref(out)),
           "iso_workspace_bytes_v")
    return out.value


def _alltoallv(name, sendbuf, send_sizes, send_displs, send_extent, recvbuf, recv_sizes, recv_displs,
               recv_extent, workspace, comm, algorithm, workspace_bytes):
    ss, sd, rs, rd = (_size_array(x) for x in (send_sizes, send_displs, recv_sizes, recv_displs))
    h = ctypes.c_void_p()
    p = lambda a: a.ctypes.data if a.size else None
    st = getattr(load_library(), name)(
        _ptr(sendbuf), p(ss), p(sd), send_extent, _ptr(recvbuf), p(rs), p(rd), recv_extent,
        _ptr(workspace), _nbytes(workspace, workspace_bytes), comm.handle, algorithm, ctypes.byref(h))
    _check(st, name)
    return Request(h.value, (sendbuf, recvbuf, workspace))


def _allgatherv(name, sendbuf, send_size, send_extent, recvbuf, recv_sizes, recv_displs, recv_extent,
                workspace, comm, algorithm, workspace_bytes):
    rs, rd = _size_array(recv_sizes), _size_array(recv_displs)
    h = ctypes.c_void_p()
    p = lambda a: a.ctypes.data if a.size else None
    st = getattr(load_library(), name)(
        _ptr(sendbuf), send_size, send_extent, _ptr(recvbuf), p(rs), p(rd), recv_extent,
        _ptr(workspace), _nbytes(workspace, workspace_bytes), comm.handle, algorithm, ctypes.byref(h))
    _check(st, name)
    return Request(h.value, (sendbuf, recvbuf, workspace))


def iso_neighbor_alltoallv_init_layout(sendbuf, send_sizes, send_displs, send_extent, recvbuf, recv_sizes,
                                       recv_displs, recv_extent, layout, workspace, comm,
                                       algorithm=ISO_ALG_COMBINED, workspace_bytes=None):
    ss, sd, rs, rd = (_size_array(x) for x in (send_sizes, send_displs, recv_sizes, recv_displs))
    h = ctypes.c_void_p()
    p = lambda a: a.ctypes.data if a.size else None
    st = load_library().iso_neighbor_alltoallv_init_layout(
        _ptr(sendbuf), p(ss), p(sd), send_extent, _ptr(recvbuf), p(rs), p(rd), recv_extent, layout,
        _ptr(workspace), _nbytes(workspace, workspace_bytes), comm.handle, algorithm, ctypes.byref(h))
    _check(st, "iso_neighbor_alltoallv_init_layout")
    return Request(h.value, (sendbuf, recvbuf, workspace))


def iso_neighbor_allgatherv_init_layout(sendbuf, send_size, send_extent, recvbuf, recv_sizes, recv_displs,
                                        recv_extent, layout, workspace, comm, algorithm=ISO_ALG_COMBINED,
                                        workspace_bytes=None):
    rs, rd = _size_array(recv_sizes), _size_array(recv_displs)
    h = ctypes.c_void_p()
    p = lambda a: a.ctypes.data if a.size else None
    st = load_library().iso_neighbor_allgatherv_init_layout(
        _ptr(sendbuf), send_size, send_extent, _ptr(recvbuf), p(rs), p(rd), recv_extent, layout,
        _ptr(workspace), _nbytes(workspace, workspace_bytes), comm.handle, algorithm, ctypes.byref(h))
    _check(st, "iso_neighbor_allgatherv_init_layout")
    return Request(h.value, (sendbuf, recvbuf, workspace))


def iso_neighbor_alltoallv_init(sendbuf, send_sizes, send_displs, send_extent, recvbuf, recv_sizes,
                                recv_displs, recv_extent, workspace, comm,
                                algorithm=ISO_ALG_COMBINED, workspace_bytes=None):
    return _alltoallv("iso_neighbor_alltoallv_init", sendbuf, send_sizes, send_displs, send_extent, recvbuf,
                      recv_sizes, recv_displs, recv_extent, workspace, comm, algorithm, workspace_bytes)


def iso_neighbor_alltoallw_init(sendbuf, send_sizes, send_displs, send_extent, recvbuf, recv_sizes,
                                recv_displs, recv_extent, workspace, comm,
                                algorithm=ISO_ALG_COMBINED, workspace_bytes=None):
    return _alltoallv("iso_neighbor_alltoallw_init", sendbuf, send_sizes, send_displs, send_extent, recvbuf,
                      recv_sizes, recv_displs, recv_extent, workspace, comm, algorithm, workspace_bytes)


def iso_neighbor_allgatherv_init(sendbuf, send_size, send_extent, recvbuf, recv_sizes, recv_displs,
                                 recv_extent, workspace, comm, algorithm=ISO_ALG_COMBINED,
                                 workspace_bytes=None):
    return _allgatherv("iso_neighbor_allgatherv_init", sendbuf, send_size, send_extent, recvbuf, recv_sizes,
                       recv_displs, recv_extent, workspace, comm, algorithm, workspace_bytes)


def iso_neighbor_allgatherw_init(sendbuf, send_size, send_extent, recvbuf, recv_sizes, recv_displs,
                                 recv_extent, workspace, comm, algorithm=ISO_ALG_COMBINED,
                                 workspace_bytes=None):
    return _allgatherv("iso_neighbor_allgatherw_init", sendbuf, send_size, send_extent, recvbuf, recv_sizes,
                       recv_displs, recv_extent, workspace, comm, algorithm, workspace_bytes)


def iso_neighbor_alltoall_noalloc(sendbuf, recvbuf, m, comm, algorithm=ISO_ALG_COMBINED, stream=None):
    """One all-to-all enqueued on `stream` with no device allocation (see iso.h)."""
    _check(load_library().iso_neighbor_alltoall_noalloc(_ptr(sendbuf), _ptr(recvbuf), m, comm.handle, algorithm,
                                                        _stream_handle(stream)), "iso_neighbor_alltoall_noalloc")


def iso_start(req, stream=None):
    """Enqueue one collective on `stream` (torch stream, raw hipStream_t value,
    or None for torch's current stream)."""
    _check(load_library().iso_start(req.handle, _stream_handle(stream)), "iso_start")


def iso_start_range(req, first, count, stream=None):
    _check(load_library().iso_start_range(req.handle, first, count, _stream_handle(stream)),
           "iso_start_range")


def iso_request_set_graph(req, enable=True):
    """enable: False / True (= ISO_GRAPH_CHAIN) or one of ISO_GRAPH_OFF / _CHAIN / _BRANCHES."""
    _check(load_library().iso_request_set_graph(req.handle, int(enable)), "iso_request_set_graph")


def iso_wait(req):
    _check(load_library().iso_wait(req.handle), "iso_wait")


def iso_request_info(req):
    info = iso_request_info_t()
    _check(load_library().iso_request_info(req.handle, ctypes.byref(info)), "iso_request_info")
    return _struct_dict(info)


def iso_request_plan(req):
    h = ctypes.c_void_p()
    _check(load_library().iso_request_plan(req.handle, ctypes.byref(h)), "iso_request_plan")
    plan = Plan(h.value, owned=False)
    plan._keepalive = req
    return plan


def iso_request_free(req):
    req.free()


def iso_error_string(status):
    return load_library().iso_error_string(status).decode()


def iso_last_hip_error():
    return load_library().iso_last_hip_error()


def iso_copy_reference(src, dst, nbytes, stream=None):
    _check(load_library().iso_copy_reference(_ptr(src), _ptr(dst), nbytes, _stream_handle(stream)),
           "iso_copy_reference")
