"""Generators of s-neighbourhoods: lists of relative coordinate vectors.

Every generator returns a Python list of s tuples of d ints, in a fixed,
documented order (the order fixes the block order in the send and receive
buffers, Section 2 of the paper).  The shapes are the ones the paper's
experiments use (Section 4): full Moore neighbourhoods, the positive-octant
asymmetric variant, Chebyshev "shales", plus a von Neumann ball and a seeded
random asymmetric neighbourhood.
"""
from itertools import product

from .blocks import mix32_int


def moore(d, r):
    """All vectors with max |c_j| <= r except the origin, lexicographic ("row")
    order; s = (2r+1)^d - 1 (Section 4, Moore neighbourhoods)."""
    return [c for c in product(range(-r, r + 1), repeat=d) if any(c)]


def von_neumann(d, r):
    """All vectors with 0 < sum |c_j| <= r, lexicographic order."""
    return [c for c in product(range(-r, r + 1), repeat=d)
            if 0 < sum(abs(x) for x in c) <= r]


def positive_octant(d, r):
    """The asymmetric Moore variant with only non-negative coordinates
    (Section 2's octant example is d=3, r=1 in another order; Section 4 uses
    d=3, r=3 with 63 neighbours).  Lexicographic order, origin excluded."""
    return [c for c in product(range(0, r + 1), repeat=d) if any(c)]


def shales(d, radii):
    """Vectors whose Chebyshev norm max |c_j| is exactly one of `radii`
    (Section 6 uses d=3, radii (3, 7): 1396 neighbours).  Lexicographic."""
    radii = sorted(set(int(x) for x in radii))
    rmax = radii[-1]
    return [c for c in product(range(-rmax, rmax + 1), repeat=d)
            if max(abs(x) for x in c) in radii]


def random_distinct(d, lo, hi, s, seed):
    """s distinct non-zero vectors, each coordinate uniform on {lo..hi}, kept
    in draw order.  Draws come from the counter-based mixer so the list is a
    pure function of (d, lo, hi, s, seed) on every platform."""
    span = hi - lo + 1
    if s > span ** d - (1 if lo <= 0 <= hi else 0):
        raise ValueError("not enough distinct non-zero vectors")
    limit = (1 << 32) - ((1 << 32) % span)      # rejection bound: exact uniformity
    out, seen, ctr = [], set(), 0
    base = mix32_int((seed ^ 0x5bd1e995) & 0xFFFFFFFF)
    while len(out) < s:
        c = []
        for _ in range(d):
            while True:
                w = mix32_int((base + ctr * 0x9E3779B1) & 0xFFFFFFFF)
                ctr += 1
                if w < limit:
                    break
            c.append(lo + w % span)
        c = tuple(c)
        if any(c) and c not in seen:
            seen.add(c)
            out.append(c)
    return out


def stencil_block_sizes(offsets, base):
    """Irregular block sizes of the paper's all-to-all-w experiment (Section 4):
    neighbour i gets base ** (d - ||C^i||_1) bytes, as in a stencil code where
    faces are larger than edges and edges larger than corners."""
    d = len(offsets[0]) if offsets else 0
    return [int(base) ** max(0, d - sum(abs(c) for c in C)) for C in offsets]


def packed_displacements(sizes, align=16):
    """Blocks laid out in neighbour order, each start rounded up to `align`
    bytes; returns (displacements, extent)."""
    displs, at = [], 0
    for n in sizes:
        at = (at + align - 1) // align * align
        displs.append(at)
        at += int(n)
    return displs, (at + align - 1) // align * align
