"""First-order prefetch/compute overlap model.  TEST INFRASTRUCTURE ONLY.

Sec. 3.1 (Eq. 1-4), App. A (operational intensity and the ridge I*), App. B (per-block FLOP
and parameter-byte formulas), App. C (numerical instantiation, Tables 1-2), Sec. 3.2
(one chunk's service time), Sec. 3.3 (partial residency scales the prefetched volume).

Units follow the paper's worked examples: MB = 1e6 bytes, GB/s = 1e9 bytes/s, TFLOP/s =
1e12.  Only with these decimal units and per-GPU FLOPs = global FLOPs / SP degree do the
three critical configurations printed in App. C come out.

The step-time closure `step_time` (sum over blocks of max(T_comp, T_pref)) and `weight_memory`
are this build's own first-order extension of the hide-or-expose condition; the paper prints
only the condition.  They are PARITY UNPINNED by the paper and are checked only through
their limits (r=0, r=1) and monotonicity in r.
"""
from __future__ import annotations

import dataclasses
from typing import Callable

# ---------------------------------------------------------------- App. B: FLOPs (global form)


def flops_dit(B, S, d, f, l_ctx):
    """DiT block: self-proj + self-attn + cross-proj + cross-attn + MLP."""
    self_proj = 8 * B * S * d * d
    self_attn = 4 * B * S * S * d
    cross_proj = 4 * B * S * d * d + 4 * B * l_ctx * d * d
    cross_attn = 4 * B * S * l_ctx * d
    mlp = 4 * B * S * d * f
    return self_proj + self_attn + cross_proj + cross_attn + mlp


def flops_double(B, S, d, f, l_ctx):
    """MM-DiT double-stream block."""
    img_proj = 8 * B * S * d * d
    txt_proj = 8 * B * l_ctx * d * d
    joint_attn = 4 * B * (S + l_ctx) ** 2 * d
    img_mlp = 4 * B * S * d * f
    txt_mlp = 4 * B * l_ctx * d * f
    return img_proj + txt_proj + joint_attn + img_mlp + txt_mlp


def flops_single(B, S, d, f, l_ctx):
    """MM-DiT single-stream block: fused linear_1, joint attention, fused linear_2."""
    n = S + l_ctx
    lin1 = 2 * B * n * d * (3 * d + f)
    attn = 4 * B * n * n * d
    lin2 = 2 * B * n * (d + f) * d
    return lin1 + attn + lin2


def flops_mmdit_avg(B, S, d, f, l_ctx, n_double, n_single):
    """Block-averaged MM-DiT FLOPs."""
    return (n_double * flops_double(B, S, d, f, l_ctx)
            + n_single * flops_single(B, S, d, f, l_ctx)) / (n_double + n_single)


# ---------------------------------------------------------------- App. B: parameter bytes

def bytes_single(d, f, beta=2):
    return beta * (7 * d * d + 2 * d * f)


def bytes_double(d, f, beta=2):
    return beta * (20 * d * d + 4 * d * f)


# ---------------------------------------------------------------- Sec. 3.1: the model

@dataclasses.dataclass(frozen=True)
class Platform:
    p_peak: float       # FLOP/s, dense bf16
    bw_h2d: float       # bytes/s per GPU
    eta_comp: float
    eta_pref: float


#: Table 1 (two H100 PCIe sharing one host root).
PAPER_PLATFORM = Platform(p_peak=756e12, bw_h2d=31.5e9, eta_comp=0.60, eta_pref=0.89)


def t_comp(flops_per_gpu, plat: Platform):
    """Eq. 1."""
    return flops_per_gpu / (plat.eta_comp * plat.p_peak)


def t_pref(b_pref, plat: Platform, resident_fraction=0.0):
    """Eq. 2; partial residency (Sec. 3.3) removes the resident share of the volume."""
    return (1.0 - resident_fraction) * b_pref / (plat.eta_pref * plat.bw_h2d)


def hidden(flops_per_gpu, b_pref, plat: Platform, resident_fraction=0.0):
    """Eq. 3: prefetch fully hidden iff T_comp >= T_pref."""
    return t_comp(flops_per_gpu, plat) >= t_pref(b_pref, plat, resident_fraction)


def f_star(b_pref, plat: Platform):
    """Eq. 4: critical compute workload."""
    return plat.eta_comp * plat.p_peak * b_pref / (plat.eta_pref * plat.bw_h2d)


def i_star(plat: Platform):
    """App. A: ridge intensity, FLOP per prefetched byte."""
    return plat.eta_comp * plat.p_peak / (plat.eta_pref * plat.bw_h2d)


def t_chunk(chunk_bytes, plat: Platform):
    """Sec. 3.2: service time of one chunk = bound on the residual stall at a pause."""
    return chunk_bytes / (plat.eta_pref * plat.bw_h2d)


def solve_increasing(g: Callable[[float], float], lo: float, hi: float, iters: int = 200) -> float:
    """Root of an increasing function by bisection."""
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        if g(mid) < 0:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def critical_config(flops_global_of: Callable[[float], float], b_pref, plat: Platform, sp_degree: int,
                    lo=1e-3, hi=1e4) -> float:
    """The configuration parameter (frames n or batch b) at which the per-GPU share of the
    block FLOPs equals F* (App. C)."""
    fs = f_star(b_pref, plat)
    return solve_increasing(lambda z: flops_global_of(z) / sp_degree - fs, lo, hi)


# ---------------------------------------------------------------- closures (parity unpinned)

def step_time(t_comp_block, b_pref, n_blocks, plat: Platform, resident_fraction=0.0):
    """Sum over blocks of max(T_comp(l), T_pref(l+1)); homogeneous stack, cyclic."""
    tp = t_pref(b_pref, plat, resident_fraction)
    return n_blocks * max(t_comp_block, tp)


def exposed_time(t_comp_block, b_pref, n_blocks, plat: Platform, resident_fraction=0.0):
    tp = t_pref(b_pref, plat, resident_fraction)
    return n_blocks * max(0.0, tp - t_comp_block)


def weight_memory(blob_bytes, n_blocks, resident_fraction):
    """Resident share of every block plus two staging slots for the streamed share."""
    return resident_fraction * n_blocks * blob_bytes + 2 * (1.0 - resident_fraction) * blob_bytes
