"""The five benchmark workloads (torus, neighbourhood, block size, content).

These are synthetic stand-ins for the paper's Moore-neighbourhood MPI
benchmarks (Section 4): same neighbourhood shapes and small-block regime, with
all p processes of the torus held as virtual ranks in one device's memory.
"""
from dataclasses import dataclass, field
from math import prod

from .neighborhoods import moore, von_neumann, random_distinct


@dataclass(frozen=True)
class Workload:
    name: str
    dims: tuple            # torus dimension sizes p_0..p_{d-1}
    offsets: tuple         # s relative coordinate vectors, block order
    m: int                 # block size in bytes
    kind: str              # "u32" | "f32" | "u8" content
    ops: tuple             # subset of ("alltoall", "allgather")
    m_sweep: tuple = field(default=())

    @property
    def p(self):
        return prod(self.dims)

    @property
    def s(self):
        return len(self.offsets)

    @property
    def d(self):
        return len(self.dims)


def _mk(name, dims, offs, m, kind, ops, sweep=()):
    return Workload(name, tuple(dims), tuple(tuple(c) for c in offs), m, kind,
                    tuple(ops), tuple(sweep))


CONFIG5_NEIGHBOURHOOD_SEED = 1606_07676

CONFIGS = (
    _mk("c1_torus8x8_moore1_m32", (8, 8), moore(2, 1), 32, "u32", ("alltoall",)),
    _mk("c2_torus32x32x32_moore1_m256", (32, 32, 32), moore(3, 1), 256, "u32",
        ("alltoall", "allgather")),
    _mk("c3_torus256x256_vn2_m1024", (256, 256), von_neumann(2, 2), 1024, "f32",
        ("alltoall",)),
    _mk("c4_torus64x64x64_moore1_m128", (64, 64, 64), moore(3, 1), 128, "u32",
        ("allgather", "alltoall"), sweep=(16, 64, 128)),
    _mk("c5_torus8x8x8x8x8_rand40_m4096", (8,) * 5,
        random_distinct(5, -3, 3, 40, CONFIG5_NEIGHBOURHOOD_SEED), 4096, "u8",
        ("alltoall", "allgather")),
)


def get_config(key):
    """Look up by 1-based index (int or digit string) or by name."""
    if isinstance(key, int) or (isinstance(key, str) and key.isdigit()):
        return CONFIGS[int(key) - 1]
    for c in CONFIGS:
        if c.name == key:
            return c
    raise KeyError(key)
