"""Counter-based generator of bf16 bit patterns.

Recipe (stands in for the actor's trained bf16 weights, which the reshard path
treats as opaque 16-bit words):

  value(seed, uid, i) = fix_nan( low16( mix64( key(seed, uid) + (i + 1) * GOLDEN ) ) )

`mix64` is the public splitmix64 output function (Steele, Lea, Flood 2014; Vigna's
reference constants).  `fix_nan` clears the lowest exponent bit of every NaN pattern
so that the data are uniform over all non-NaN bf16 encodings (infinities, zeros and
subnormals stay): float-typed comparisons of the buffers can then never be confused
by NaN != NaN, although all checks in this repository compare integers anyway.

Three implementations of the same function: pure Python (one element), numpy
(host arrays) and torch int64 ops (any torch device; used to fill tens of GB in HBM
without a host round trip).  tests/test_seeded_inputs.py checks them against each
other and against hand-computed splitmix64 outputs.
"""
from __future__ import annotations

import numpy as np

_M64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

# Stream ids of the training-layout tensors.  Pure naming: no shapes, no offsets.
KIND_IDS = {
    "embed": 1, "ln1": 2, "qkv": 3, "o": 4, "ln2": 5, "gate_up": 6, "down": 7,
    "lnf": 8, "head": 9,
}


def config_seed(config_index: int) -> int:
    """Seed of BASELINE config `config_index` (0-based)."""
    return 0x240919256 + int(config_index)


def tensor_uid(kind: str, layer: int, tp_index: int) -> int:
    """Stream id of one training-shard tensor.

    `layer` is the global layer number (0 for embed/lnf/head); `tp_index` is the
    tensor-parallel index of the shard for TP-sharded tensors and MUST be 0 for
    tensors replicated over TP (the caller decides which are).  The data-parallel
    index is deliberately not part of the id: DP replicas hold identical weights.
    """
    return KIND_IDS[kind] + 16 * (int(layer) + 1) + (1 << 24) * int(tp_index)


def _mix64(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, uid: int) -> int:
    """64-bit key of stream `uid` under `seed` (host scalar arithmetic)."""
    return _mix64((int(seed) & _M64) ^ ((int(uid) * GOLDEN) & _M64))


def _fix_nan_scalar(b: int) -> int:
    if (b & 0x7F80) == 0x7F80 and (b & 0x007F):
        b ^= 0x0080
    return b


def bits16_scalar(key: int, index: int) -> int:
    """One element, plain Python integers."""
    return _fix_nan_scalar(_mix64(key + (int(index) + 1) * GOLDEN) & 0xFFFF)


def bits16_numpy(key: int, start: int, count: int) -> np.ndarray:
    """Elements start .. start+count-1 of stream `key` as uint16."""
    with np.errstate(over="ignore"):
        i = np.arange(start + 1, start + 1 + count, dtype=np.uint64)
        z = i * np.uint64(GOLDEN) + np.uint64(key)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_C1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_C2)
        z = z ^ (z >> np.uint64(31))
    b = (z & np.uint64(0xFFFF)).astype(np.uint16)
    nan = ((b & np.uint16(0x7F80)) == np.uint16(0x7F80)) & ((b & np.uint16(0x007F)) != 0)
    return np.where(nan, b ^ np.uint16(0x0080), b)


def _s64(x: int) -> int:
    """Two's-complement int64 view of an unsigned 64-bit constant."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def bits16_torch(key: int, start: int, count: int, device="cpu"):
    """Same stream as `bits16_numpy`, as an int16 torch tensor on `device`.

    int64 arithmetic wraps modulo 2**64 exactly like uint64; logical right shifts
    are an arithmetic shift followed by a mask of the bits shifted in.
    """
    import torch

    def lsr(z, s):
        return (z >> s) & ((1 << (64 - s)) - 1)

    i = torch.arange(start + 1, start + 1 + count, dtype=torch.int64, device=device)
    z = i * _s64(GOLDEN) + _s64(key)
    z = (z ^ lsr(z, 30)) * _s64(_C1)
    z = (z ^ lsr(z, 27)) * _s64(_C2)
    z = z ^ lsr(z, 31)
    b = z & 0xFFFF
    nan = ((b & 0x7F80) == 0x7F80) & ((b & 0x007F) != 0)
    b = torch.where(nan, b ^ 0x0080, b)
    # 0..65535 -> the int16 with the same bit pattern
    return torch.where(b >= 0x8000, b - 0x10000, b).to(torch.int16)


def fill_regions_numpy(buf_u16: np.ndarray, regions, seed: int) -> None:
    """Fill regions of a uint16 host array.

    `regions` is an iterable of (elem_offset, n_elems, uid): region k receives
    elements 0..n_elems-1 of stream `uid`.  Bytes outside the regions are untouched.
    """
    for off, n, uid in regions:
        buf_u16[off:off + n] = bits16_numpy(stream_key(seed, uid), 0, n)


def fill_regions_torch(buf_i16, regions, seed: int, chunk: int = 1 << 25) -> None:
    """Same as `fill_regions_numpy` for a 1-D int16 torch tensor on any device."""
    for off, n, uid in regions:
        key = stream_key(seed, uid)
        done = 0
        while done < n:
            c = min(chunk, n - done)
            buf_i16[off + done:off + done + c] = bits16_torch(key, done, c, buf_i16.device)
            done += c
