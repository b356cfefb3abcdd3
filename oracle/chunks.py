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


# ---------------------------------------------------------------- blob layout (this build's own)

def blob_layout(cfg):
    """[(name, offset, rows, cols)] of one block's bf16 tensors inside its blob.

    The paper fixes no layout.  This build packs a block's parameters in the order the block
    consumes them, small vectors ahead of the matrix they go with, every tensor on a 256-byte
    boundary and the blob padded to one, so that a prefix of chunks is a prefix of the
    computation (Sec. 3.2).  Matrices are [out_features, in_features].  A double-stream block
    lists the text stream before the image stream inside every stage."""
    d, f, hd = cfg.d, cfg.f, cfg.head_dim
    norms = lambda pre: ([(pre + "q_norm", 1, hd), (pre + "k_norm", 1, hd)] if cfg.qk_rmsnorm else [])
    if cfg.kind == 0:      # single-stream
        ts = [("b_mod", 1, 3 * d), ("w_mod", 3 * d, d), ("b1", 1, 3 * d + f)] + norms("") + \
             [("w1", 3 * d + f, d), ("b2", 1, d), ("w2", d, d + f)]
    elif cfg.kind == 1:    # DiT with cross-attention
        ts = [("b_mod", 1, 6 * d), ("w_mod", 6 * d, d), ("b_qkv", 1, 3 * d)] + norms("") + \
             [("w_qkv", 3 * d, d), ("b_o", 1, d), ("w_o", d, d), ("ln_c_w", 1, d), ("ln_c_b", 1, d), ("b_cq", 1, d)] + \
             norms("c") + \
             [("w_cq", d, d), ("b_ckv", 1, 2 * d), ("w_ckv", 2 * d, d), ("b_co", 1, d), ("w_co", d, d),
              ("b_up", 1, f), ("w_up", f, d), ("b_down", 1, d), ("w_down", d, f)]
    else:                  # double-stream
        ts = []
        for s in ("txt_", "img_"):
            ts += [(s + "b_mod", 1, 6 * d), (s + "w_mod", 6 * d, d)]
        for s in ("txt_", "img_"):
            ts += [(s + "b_qkv", 1, 3 * d)] + norms(s) + [(s + "w_qkv", 3 * d, d)]
        for s in ("txt_", "img_"):
            ts += [(s + "b_o", 1, d), (s + "w_o", d, d)]
        for s in ("txt_", "img_"):
            ts += [(s + "b_up", 1, f), (s + "w_up", f, d), (s + "b_down", 1, d), (s + "w_down", d, f)]
    out, off = [], 0
    for name, rows, cols in ts:
        off = -(-off // 256) * 256
        out.append((name, off, rows, cols))
        off += 2 * rows * cols
    return out, -(-off // 256) * 256
