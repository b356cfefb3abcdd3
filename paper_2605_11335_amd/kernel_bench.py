"""Single-kernel microbenchmarks through the C ABI (linear layers, attention) plus a plain
device-to-device copy of known size, used to calibrate hardware byte counters.

    python -m paper_2605_11335_amd.kernel_bench linear 2304x21504x3072 [iters]
    python -m paper_2605_11335_amd.kernel_bench linear_residual 2304x3072x15360 [iters]
    python -m paper_2605_11335_amd.kernel_bench attention 12x4608x128 [iters]
    python -m paper_2605_11335_amd.kernel_bench copy 536870912 [iters]      # bytes
    python -m paper_2605_11335_amd.kernel_bench checksum 283183616 [iters]  # bytes (a C2 blob)
    python -m paper_2605_11335_amd.kernel_bench mfma_rate 20000 [iters]     # MFMAs on registers only
    python -m paper_2605_11335_amd.kernel_bench mix_rate 20000 [iters]      # MFMAs beside LDS reads and VALU work

Timing uses events on the current stream; inputs are seeded N(0,1) activations and N(0,0.02)
weights in bf16.  The GEMM benchmarks rotate over enough operand sets that consecutive launches
never find their operands in the 256 MB last-level cache: inside a block every weight byte is read
once per step, cold, and tile shapes rank differently hot and cold.
"""
from __future__ import annotations

import sys

import torch

from . import binding as B

DEV = "cuda:0"


def timeit(fn, iters):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(iters):
        fn()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / iters


def main(argv):
    which, shape = argv[1], argv[2]
    iters = int(argv[3]) if len(argv) > 3 else 20
    torch.manual_seed(0)
    if which in ("linear", "linear_residual"):
        M, N, K = (int(v) for v in shape.split("x"))
        sets = max(2, -(-(1 << 30) // (2 * K * (M + N))))        # operands of all sets together > 1 GiB
        A = [torch.randn(M, K, device=DEV).to(torch.bfloat16) for _ in range(sets)]
        W = [(torch.randn(N, K, device=DEV) * 0.02).to(torch.bfloat16) for _ in range(sets)]
        turn = [0]

        def nxt():
            turn[0] = (turn[0] + 1) % sets
            return turn[0]

        if which == "linear":
            out = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
            ms = timeit(lambda: B.cf_op_linear(A[nxt()], W[turn[0]], 0, -1, M, N, K, out), iters)
        else:
            resid = torch.randn(M, N, device=DEV)
            gate = torch.randn(N, device=DEV)
            y = torch.empty(M, N, device=DEV)
            ms = timeit(lambda: B.cf_op_linear_residual(A[nxt()], W[turn[0]], 0, -1, M, N, K, resid, gate, y), iters)
        print(f"{which} {M}x{N}x{K} ({sets} operand sets in turn): {ms:.4f} ms  {2 * M * N * K / ms / 1e9:.1f} TFLOP/s")
    elif which == "attention":
        H, N, hd = (int(v) for v in shape.split("x"))
        npad = (N + 63) // 64 * 64
        Q = torch.randn(H, N, hd, device=DEV).to(torch.bfloat16)
        K_ = torch.randn(H, N, hd, device=DEV).to(torch.bfloat16)
        Vt = torch.zeros(H, hd, npad, device=DEV, dtype=torch.bfloat16)
        Vt[:, :, :N] = torch.randn(H, hd, N, device=DEV).to(torch.bfloat16)
        O = torch.empty(H, N, hd, dtype=torch.bfloat16, device=DEV)
        ms = timeit(lambda: B.cf_op_attention(Q, K_, Vt, O, H, N, N, npad, hd), iters)
        print(f"attention H={H} N={N} hd={hd}: {ms:.4f} ms  {4 * H * N * N * hd / ms / 1e9:.1f} TFLOP/s")
    elif which == "copy":
        n = int(shape)
        src = torch.empty(n, dtype=torch.uint8, device=DEV).random_(0, 255)
        dst = torch.empty_like(src)
        ms = timeit(lambda: dst.copy_(src), iters)
        print(f"copy {n} bytes: {ms:.4f} ms  {2 * n / ms / 1e6:.1f} GB/s (read + write)")
    elif which == "checksum":
        n = int(shape) // 8 * 8
        data = torch.empty(n, dtype=torch.uint8, device=DEV).random_(0, 255)
        ms = timeit(lambda: B.cf_op_checksum(data, n, 0), iters)       # reads the result back: a host sync per call
        print(f"checksum {n} bytes: {ms:.4f} ms  {n / ms / 1e6:.1f} GB/s (read)")
    elif which == "mfma_rate":
        n = int(shape)
        out = torch.empty(256 * 256, dtype=torch.float32, device=DEV)
        flops = 256 * 4 * n * 16 * 32768.0
        for rnd, what in ((False, "one pair of small-valued fragments repeated"), (True, "16 pairs of unit-variance random fragments")):
            ms = timeit(lambda: B.cf_op_mfma_rate(n, rnd, out), iters)
            print(f"mfma_rate {n} x 16 MFMAs per wave, 1024 waves, {what}: {ms:.4f} ms  {flops / ms / 1e9:.1f} TFLOP/s "
                  f"({flops / ms / 1e9 / 2500 * 100:.1f} % of the published 2500; implied clock {flops / ms / 1e9 / 2500 * 2.4:.2f} GHz)")
    elif which == "mix_rate":
        n = int(shape)
        out = torch.empty(256 * 512, dtype=torch.float32, device=DEV)
        mixes = [(4, 0, 0, 0), (8, 0, 0, 0), (4, 8, 0, 0), (8, 8, 0, 0), (8, 16, 0, 0), (8, 0, 2, 0), (8, 0, 4, 0), (8, 0, 2, 1),
                 (8, 0, 4, 1), (8, 16, 4, 1), (8, 16, 2, 1), (8, 8, 4, 1), (8, 8, 2, 1), (4, 8, 4, 1), (4, 8, 2, 1), (4, 16, 4, 1)]
        base = None
        for waves, reads, valu, exps in mixes:
            it = n * 8 // waves                                     # the same number of MFMAs per CU in every row
            ms = timeit(lambda: B.cf_op_mix_rate(it, waves, reads, valu, exps, out), iters)
            tf = 256 * waves * it * 16 * 32768.0 / ms / 1e9
            base = base or tf
            print(f"mix_rate waves/CU {waves}  LDS reads per 16 MFMAs {reads:2d}  VALU per MFMA {valu}  exp2 per MFMA {exps}: "
                  f"{ms:8.3f} ms  {tf:7.1f} TFLOP/s  ({tf / base * 100:5.1f} % of MFMAs alone)")
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv)
