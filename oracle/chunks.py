"""Chunk arithmetic and the streamed-bytes checksum.  TEST INFRASTRUCTURE ONLY.

Sec. 3.2: a layer's parameters are cut into fixed-size chunks (the last one may be short);
chunking never changes the total volume.  Sec. 3.3: residency is decided per chunk; 0 %
is full offload, 100 % is no offload.  This build keeps a prefix of each block's chunks
resident and rounds r*n_chunks half up; the paper leaves both choices open.

The checksum is this build's own definition (the paper has none): the blob is read as
little-endian 64-bit words; word i (index counted from the start of the BLOB) contributes
mix(word XOR (i+1)*GOLDEN) and contributions add modulo 2^64, where mix is the splitmix64
finaliser.  Position-dependent, order-independent to evaluate.
"""
from __future__ import annotations

import numpy as np

GOLDEN = 0x9E3779B97F4A7C15
M1 = 0xBF58476D1CE4E5B9
M2 = 0x94D049BB133111EB
MASK = (1 << 64) - 1


def chunk_bounds(blob_bytes: int, chunk_bytes: int):
    """[(begin, end)) byte ranges of the chunks of one blob."""
    return [(b, min(b + chunk_bytes, blob_bytes)) for b in range(0, blob_bytes, chunk_bytes)]


def n_resident(n_chunks: int, r: float) -> int:
    return int(np.floor(r * n_chunks + 0.5))


def resident_bytes(blob_bytes: int, chunk_bytes: int, r: float) -> int:
    cb = chunk_bounds(blob_bytes, chunk_bytes)
    k = n_resident(len(cb), r)
    return cb[k - 1][1] if k > 0 else 0


def _mix_py(z: int) -> int:
    z &= MASK
    z = ((z ^ (z >> 30)) * M1) & MASK
    z = ((z ^ (z >> 27)) * M2) & MASK
    return z ^ (z >> 31)


def checksum_words_py(data: bytes, first_word_index: int) -> int:
    """Reference in plain Python integers (slow; for pins and small inputs)."""
    assert len(data) % 8 == 0
    acc = 0
    for j in range(len(data) // 8):
        w = int.from_bytes(data[8 * j:8 * j + 8], "little")
        acc = (acc + _mix_py(w ^ (((first_word_index + j + 1) * GOLDEN) & MASK))) & MASK
    return acc


def checksum_words(data: np.ndarray, first_word_index: int) -> int:
    """Same function, vectorised over uint64 (wrap-around arithmetic)."""
    w = np.ascontiguousarray(data).view(np.uint8).reshape(-1).view("<u8")
    with np.errstate(over="ignore"):
        idx = (np.arange(len(w), dtype=np.uint64) + np.uint64(first_word_index + 1)) * np.uint64(GOLDEN)
        z = w ^ idx
        z = (z ^ (z >> np.uint64(30))) * np.uint64(M1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(M2)
        z = z ^ (z >> np.uint64(31))
        return int(z.sum(dtype=np.uint64))


def chunk_checksums(blob: np.ndarray, chunk_bytes: int):
    """Per-chunk checksums of a host blob (uint8 array)."""
    b = np.ascontiguousarray(blob).view(np.uint8).reshape(-1)
    return [checksum_words(b[s:e], s // 8) for s, e in chunk_bounds(len(b), chunk_bytes)]
