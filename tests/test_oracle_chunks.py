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
