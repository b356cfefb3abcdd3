"""The entry point that allocates nothing (cf_op_checksum_noalloc) against the allocating one
(cf_op_checksum) and the oracle's plain-integer definition, through the C ABI: bit-exact, on calls
in a row that share the library's fixed partial-sum array, each smaller than the one before."""
import numpy as np
import pytest
import torch

from oracle import chunks as och
from paper_2605_11335_amd import binding as B
from tests.util import need_gpu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
WG_BYTES = 4096 * 8          # bytes one workgroup of the partial-sum kernel covers


def run_case(nbytes, first, seed):
    rng = np.random.default_rng(seed)
    data = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
    dev = torch.from_numpy(data).to(DEV) if nbytes else torch.zeros(8, dtype=torch.uint8, device=DEV)
    out = torch.full((1,), -1, dtype=torch.int64, device=DEV)          # stale value that must be overwritten
    torch.cuda.synchronize()
    B.cf_op_checksum_noalloc(dev, nbytes, first, out)
    torch.cuda.synchronize()
    got = int(out.cpu().numpy().view(np.uint64)[0])
    assert got == B.cf_op_checksum(dev, nbytes, first), (nbytes, first)
    assert got == och.checksum_words(data, first), (nbytes, first)


def test_no_alloc_checksum_equals_allocating_one_on_shrinking_inputs():
    need_gpu()
    # several workgroups with a ragged last one; then fewer workgroups; a single partly filled one; one word;
    # nothing at all: every call leaves partial sums of the larger call before it further up in the array
    sizes = [37 * WG_BYTES + 8 * 123, 5 * WG_BYTES + 8 * 4095, WG_BYTES, 8 * 1001, 8, 0]
    for i, n in enumerate(sizes):
        print(f"checksum_noalloc: {n} bytes", flush=True)
        run_case(n, 12345 + 7 * i, seed=n + 1)


def test_no_alloc_checksum_at_the_size_limit_of_a_chunk():
    need_gpu()
    n = 256 << 20                       # the largest chunk size of the sweep, 8192 workgroups
    print(f"checksum_noalloc: {n} bytes", flush=True)
    data = torch.randint(0, 256, (n,), dtype=torch.uint8, device=DEV)
    out = torch.zeros(1, dtype=torch.int64, device=DEV)
    B.cf_op_checksum_noalloc(data, n, 3, out)
    torch.cuda.synchronize()
    assert int(out.cpu().numpy().view(np.uint64)[0]) == B.cf_op_checksum(data, n, 3)
    run_case(8 * 77, 0, seed=5)         # and a small one right after it


def test_no_alloc_checksum_rejects_what_its_array_cannot_cover():
    need_gpu()
    z = torch.zeros(16, dtype=torch.uint8, device=DEV)
    out = torch.zeros(1, dtype=torch.int64, device=DEV)
    with pytest.raises(B.ChunkflowError) as e:
        B.cf_op_checksum_noalloc(z, (1 << 30) + 8, 0, out)
    assert e.value.code == B.CF_ERR_ARG and "exceed" in str(e.value)
    with pytest.raises(B.ChunkflowError):
        B.cf_op_checksum_noalloc(z, 12, 0, out)            # not whole words
    with pytest.raises(B.ChunkflowError):
        B.cf_op_checksum_noalloc(z, 8, 0, None)
