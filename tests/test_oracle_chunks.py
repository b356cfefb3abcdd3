import numpy as np
import pytest

from oracle import chunks as ch


def test_splitmix64_known_answer():
    # first output of the published splitmix64 generator seeded with 0
    assert ch._mix_py(ch.GOLDEN) == 0xE220A8397B1DCDAF


def test_vectorised_checksum_equals_plain_integers():
    rng = np.random.default_rng(1)
    data = rng.integers(0, 256, size=8 * 1000, dtype=np.uint8)
    assert ch.checksum_words(data, 0) == ch.checksum_words_py(data.tobytes(), 0)
    assert ch.checksum_words(data[80:], 10) == ch.checksum_words_py(data[80:].tobytes(), 10)


def test_checksum_is_position_sensitive_and_additive():
    rng = np.random.default_rng(2)
    data = rng.integers(0, 256, size=8 * 64, dtype=np.uint8)
    swapped = data.copy()
    swapped[:8], swapped[8:16] = data[8:16], data[:8]
    assert ch.checksum_words(data, 0) != ch.checksum_words(swapped, 0)
    whole = ch.checksum_words(data, 0)
    parts = (ch.checksum_words(data[:256], 0) + ch.checksum_words(data[256:], 32)) % (1 << 64)
    assert whole == parts


@pytest.mark.parametrize("blob,chunk", [(7_864_320, 1_966_080), (283_115_520, 16 << 20), (1000 * 256, 7 * 256)])
def test_chunking_keeps_total_volume(blob, chunk):
    cb = ch.chunk_bounds(blob, chunk)
    assert cb[0][0] == 0 and cb[-1][1] == blob
    assert all(a[1] == b[0] for a, b in zip(cb, cb[1:]))
    assert all(e - s == chunk for s, e in cb[:-1]) and 0 < cb[-1][1] - cb[-1][0] <= chunk
    assert sum(e - s for s, e in cb) == blob


def test_residency_limits():
    blob, chunk = 283_115_520, 16 << 20
    assert ch.resident_bytes(blob, chunk, 0.0) == 0
    assert ch.resident_bytes(blob, chunk, 1.0) == blob
    vals = [ch.resident_bytes(blob, chunk, r) for r in np.linspace(0, 1, 21)]
    assert vals == sorted(vals)
    assert ch.n_resident(8, 0.25) == 2 and ch.n_resident(17, 0.5) == 9 and ch.n_resident(4, 0.1) == 0


def test_blob_layout_against_offsets_worked_by_hand():
    """The layout rule (consumption order, every tensor on a 256-byte boundary, blob padded to one)
    applied by hand to two configurations; the byte counts of the matrices are App. B's
    beta (7 d^2 + 2 d f) = 7,864,320 (d=512, f=2048) and 283,115,520 (d=3072, f=12288)."""
    from types import SimpleNamespace
    toy = SimpleNamespace(kind=0, d=512, f=2048, head_dim=64, qk_rmsnorm=False)
    lay, blob = ch.blob_layout(toy)
    assert lay == [("b_mod", 0, 1, 1536),                 # 3072 bytes
                   ("w_mod", 3072, 1536, 512),            # + 1,572,864
                   ("b1", 1_575_936, 1, 3584),            # + 7168
                   ("w1", 1_583_104, 3584, 512),          # + 3,670,016
                   ("b2", 5_253_120, 1, 512),             # + 1024
                   ("w2", 5_254_144, 512, 2560)]          # + 2,621,440
    assert blob == 7_875_584
    assert sum(2 * r * c for _, _, r, c in lay if r > 1) == 7_864_320
    flux = SimpleNamespace(kind=0, d=3072, f=12288, head_dim=128, qk_rmsnorm=True)
    lay, blob = ch.blob_layout(flux)
    # the two 256-byte norm weights are the only tensors that need padding (128 elements = 256 bytes: none)
    assert lay == [("b_mod", 0, 1, 9216), ("w_mod", 18_432, 9216, 3072), ("b1", 56_641_536, 1, 21504),
                   ("q_norm", 56_684_544, 1, 128), ("k_norm", 56_684_800, 1, 128),
                   ("w1", 56_685_056, 21504, 3072), ("b2", 188_805_632, 1, 3072), ("w2", 188_811_776, 3072, 15360)]
    assert blob == 283_183_616
    assert sum(2 * r * c for _, _, r, c in lay if r > 1) == 283_115_520
    # a tensor whose size is not a multiple of 256 bytes pushes its successor to the next boundary
    odd = SimpleNamespace(kind=0, d=256, f=64, head_dim=64, qk_rmsnorm=True)
    lay, blob = ch.blob_layout(odd)
    by = {n: o for n, o, _, _ in lay}
    assert by["q_norm"] + 256 == by["k_norm"] and by["k_norm"] + 256 == by["w1"]      # 128-byte vectors, padded
    assert blob % 256 == 0
