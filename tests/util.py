"""Shared helpers for the GPU parity tests (no method arithmetic beyond error metrics)."""
import numpy as np
import torch

import workload as wl


def need_gpu():
    import pytest
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def bf16_round(a):
    """float array -> nearest bf16 values, as float32, plus the bit patterns."""
    bits = wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))
    return wl.bf16_bits_to_f32(bits), bits


def dev_bits(bits, dev="cuda:0"):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev)


def host_bits(t):
    return t.cpu().numpy().view(np.uint16)


def bits_to_f64(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def rel_l2(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30))


def max_abs(got, ref):
    return float(np.abs(np.asarray(got, np.float64) - np.asarray(ref, np.float64)).max())


def assert_bf16_close(got_bits, ref, extra_abs=0.0, ulps=1.0):
    """Every element within `ulps` bf16 ulps of the exact value (plus an absolute floor)."""
    got = bits_to_f64(got_bits)
    ref = np.asarray(ref, np.float64)
    tol = ulps * 2.0 ** -8 * np.abs(ref) * 2 + extra_abs
    bad = np.abs(got - ref) > tol
    assert not bad.any(), f"{bad.sum()} of {bad.size} off; worst {np.abs(got - ref).max():.3e} " \
                          f"at ref {ref.reshape(-1)[np.abs(got - ref).argmax()]:.4f}"
