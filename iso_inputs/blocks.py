"""Counter-based block contents: every 32-bit word of every block is a pure
function of (seed, rank, slot, word index).

Because the content of a block can be regenerated from its indices alone, an
expected receive buffer can be produced and compared in rank chunks without
ever holding the whole send buffer, and any mis-routed block, swapped slot or
shift inside a block changes at least one word: each stage below is a
bijection of the 32-bit state for fixed other indices, so two index tuples that
differ in exactly one index never give the same word.

Two implementations of the same function live here on purpose: numpy (host)
and torch (any device, used to fill large device buffers without a PCIe
copy).  `tests/test_inputs.py` checks that they agree bit for bit.
"""
import numpy as np

_M1 = 0x7FEB352D
_M2 = 0x846CA68B
_K_SEED = 0x9E3779B9
_K_SLOT = 0x85EBCA6B
_K_SLOT_ADD = 0x27D4EB2F
_K_ELEM = 0xC2B2AE35
ALLGATHER_TWEAK = 0xA5A5A5A5      # allgather blocks: seed ^ tweak, slot 0
_MASK = 0xFFFFFFFF


def mix32_int(x):
    """The 32-bit finaliser on a Python int (xor-shift / odd-multiply rounds;
    each step is invertible modulo 2^32)."""
    x &= _MASK
    x ^= x >> 16
    x = (x * _M1) & _MASK
    x ^= x >> 15
    x = (x * _M2) & _MASK
    x ^= x >> 16
    return x


def mix32(x):
    """Same finaliser on a numpy uint32 array (wraps modulo 2^32)."""
    x = np.asarray(x, dtype=np.uint32).copy()
    x ^= x >> np.uint32(16)
    x *= np.uint32(_M1)
    x ^= x >> np.uint32(15)
    x *= np.uint32(_M2)
    x ^= x >> np.uint32(16)
    return x


def _to_kind_np(words, kind):
    if kind in ("u32", "u8"):
        return words
    if kind == "f32":
        # top 24 bits k -> k * 2^-23 - 1, exact in binary32, in [-1, 1)
        k = (words >> np.uint32(8)).astype(np.float32)
        f = k * np.float32(2.0 ** -23) - np.float32(1.0)
        return f.view(np.uint32)
    raise ValueError("kind must be 'u32', 'f32' or 'u8'")


def block_words(seed, ranks, slots, n_words, kind="u32"):
    """uint32 array of shape broadcast(ranks, slots).shape + (n_words,)."""
    ranks = np.asarray(ranks, dtype=np.int64)
    slots = np.asarray(slots, dtype=np.int64)
    h = mix32_int((seed + _K_SEED) & _MASK)
    hr = mix32(np.uint32(h) ^ ranks.astype(np.uint32))
    hs = mix32(hr + slots.astype(np.uint32) * np.uint32(_K_SLOT) + np.uint32(_K_SLOT_ADD))
    e = np.arange(n_words, dtype=np.uint32) * np.uint32(_K_ELEM)
    return _to_kind_np(mix32(hs[..., None] ^ e), kind)


def _as_bytes_np(words, m, kind="u32"):
    if kind == "u8":                 # one draw per byte: its low 8 bits
        return np.ascontiguousarray(words.astype(np.uint8))
    b = np.ascontiguousarray(words).view(np.uint8)
    return b[..., :m] if b.shape[-1] != m else b


def _n_draws(m, kind):
    """Mixer values one block of m bytes takes: one per 32-bit word, or one per byte
    for 'u8' content (uniform random bytes, each byte its own draw)."""
    return m if kind == "u8" else (m + 3) // 4


def block_bytes(seed, ranks, slots, m, kind="u32"):
    """uint8 array broadcast(ranks, slots).shape + (m,): the first m bytes
    (little-endian words) of each indexed block; kind 'u8': byte e is the low
    byte of the mixer value for element e."""
    if kind == "f32" and m % 4:
        raise ValueError("f32 blocks need m % 4 == 0")
    return _as_bytes_np(block_words(seed, ranks, slots, _n_draws(m, kind), kind), m, kind)


def alltoall_send(seed, p, s, m, kind="u32", rank_lo=0, rank_hi=None):
    """Host send buffer rows [rank_lo, rank_hi) of an all-to-all: uint8 array of
    shape (rows, s, m); block (R, i) holds the words for (seed, R, i, .)."""
    rank_hi = p if rank_hi is None else rank_hi
    if kind == "f32" and m % 4:
        raise ValueError("f32 blocks need m % 4 == 0")
    ranks = np.arange(rank_lo, rank_hi, dtype=np.int64)[:, None]
    slots = np.arange(s, dtype=np.int64)[None, :]
    return _as_bytes_np(block_words(seed, ranks, slots, _n_draws(m, kind), kind), m, kind)


def allgather_send(seed, p, m, kind="u32", rank_lo=0, rank_hi=None):
    """Host send buffer rows of an allgather: uint8 (rows, m); one block per rank."""
    rank_hi = p if rank_hi is None else rank_hi
    ranks = np.arange(rank_lo, rank_hi, dtype=np.int64)
    w = block_words(seed ^ ALLGATHER_TWEAK, ranks, np.zeros_like(ranks), _n_draws(m, kind), kind)
    return _as_bytes_np(w, m, kind)


# --------------------------------------------------------------------------
# torch twin (int32 two's-complement arithmetic == uint32 modulo 2^32)
# --------------------------------------------------------------------------

def _s32(c):
    c &= _MASK
    return c - (1 << 32) if c >= (1 << 31) else c


def _mix32_t(x):
    x = x ^ ((x >> 16) & 0xFFFF)
    x = x * _s32(_M1)
    x = x ^ ((x >> 15) & 0x1FFFF)
    x = x * _s32(_M2)
    x = x ^ ((x >> 16) & 0xFFFF)
    return x


def block_words_torch(seed, ranks, slots, n_words, kind="u32"):
    """int32 tensor (same bit patterns as `block_words`) on ranks.device.
    `ranks` and `slots` are integer tensors that broadcast together."""
    import torch
    dev = ranks.device
    h = _s32(mix32_int((seed + _K_SEED) & _MASK))
    hr = _mix32_t(ranks.to(torch.int32) ^ h)
    hs = _mix32_t(hr + slots.to(torch.int32) * _s32(_K_SLOT) + _s32(_K_SLOT_ADD))
    e = torch.arange(n_words, dtype=torch.int32, device=dev) * _s32(_K_ELEM)
    w = _mix32_t(hs[..., None] ^ e)
    if kind in ("u32", "u8"):
        return w
    if kind == "f32":
        k = ((w >> 8) & 0xFFFFFF).to(torch.float32)
        return (k * (2.0 ** -23) - 1.0).view(torch.int32)
    raise ValueError("kind must be 'u32', 'f32' or 'u8'")


def _as_bytes_t(words, m, kind="u32"):
    import torch
    if kind == "u8":
        return (words & 0xFF).to(torch.uint8)
    b = words.contiguous().view(torch.uint8)
    return b[..., :m].contiguous() if b.shape[-1] != m else b


def block_bytes_torch(seed, ranks, slots, m, kind="u32"):
    """torch twin of `block_bytes` (uint8 tensor on ranks.device)."""
    return _as_bytes_t(block_words_torch(seed, ranks, slots, _n_draws(m, kind), kind), m, kind)


def alltoall_send_torch(seed, p, s, m, kind="u32", device="cpu", out=None,
                        rank_chunk=4096):
    """uint8 tensor (p, s, m) on `device`, filled chunk by chunk."""
    import torch
    if out is None:
        out = torch.empty((p, s, m), dtype=torch.uint8, device=device)
    slots = torch.arange(s, dtype=torch.int64, device=device)[None, :]
    if kind == "u8":
        rank_chunk = max(1, rank_chunk // 8)       # four bytes of intermediate per byte of output
    for lo in range(0, p, rank_chunk):
        hi = min(p, lo + rank_chunk)
        ranks = torch.arange(lo, hi, dtype=torch.int64, device=device)[:, None]
        out[lo:hi] = _as_bytes_t(block_words_torch(seed, ranks, slots, _n_draws(m, kind), kind), m, kind)
    return out


def allgather_send_torch(seed, p, m, kind="u32", device="cpu"):
    import torch
    ranks = torch.arange(p, dtype=torch.int64, device=device)
    w = block_words_torch(seed ^ ALLGATHER_TWEAK, ranks, torch.zeros_like(ranks),
                          _n_draws(m, kind), kind)
    return _as_bytes_t(w, m, kind)
