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
their limits (r=0, r=1) and monotonicity in r.  The chunk-level walk (`segment_shares`,
`simulate_step`) is this build's own as well: its booking rule is pinned on layouts worked by
hand, its recurrence on the first-order limits and a two-block case worked by hand; what it
predicts is judged against measurement.
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


# ---------------------------------------------------------------- chunk-level walk (parity unpinned)

def segment_shares(cfg, layout, blob_bytes, chunk_bytes):
    """Share of one block's compute that each chunk completes (sums to 1).

    A weight matrix contributes its App. B term, 2 * rows_of_activations * out * in FLOPs.  The
    scheduler runs a linear layer in panels of whole row groups, a group being as many output
    features as it takes, in 256-wide tiles, to give 256 tiles together with the 256-row token
    tiles (a launch that covers the chip less than once is no faster than one that covers it
    once); a group is booked on the chunk that holds its last byte.  The modulation matrix
    multiplies a single vector and goes 8 rows at a time.  The joint attention term
    (4 * H_local * N^2 * hd for this rank's heads) is booked on the chunk that completes the QKV
    projection, the DiT block's cross-attention term (4 * H * n_local * L_ctx * hd) on the chunk
    that completes the context K/V projection."""
    n_chunks = -(-blob_bytes // chunk_bytes)
    seg = [0.0] * n_chunks
    batch = getattr(cfg, "batch", 1)        # App. B: every term is linear in the batch size B
    nl = batch * cfg.n_total / cfg.sp_degree
    tl = batch * cfg.n_txt / cfg.sp_degree
    for name, off, rows, cols in layout:
        if rows == 1:
            continue
        if name.endswith("w_mod"):
            act, group = float(batch), 8
        else:
            if cfg.kind == 1:
                act = batch * cfg.l_ctx if name == "w_ckv" else nl
            elif cfg.kind == 2:
                act = tl if name.startswith("txt_") else nl - tl
            else:
                act = nl
            token_tiles = max(1, -(-int(act) // 256))
            group = 256 * -(-256 // token_tiles)
        for r0 in range(0, rows, group):
            r1 = min(rows, r0 + group)
            seg[(off + r1 * 2 * cols - 1) // chunk_bytes] += 2.0 * act * (r1 - r0) * cols
        end = off + 2 * rows * cols
        if name in ("w1", "w_qkv", "img_w_qkv"):
            seg[(end - 1) // chunk_bytes] += 4.0 * batch * (cfg.n_heads / cfg.sp_degree) * cfg.n_total * cfg.n_total * cfg.head_dim
        if name == "w_ckv":
            seg[(end - 1) // chunk_bytes] += 4.0 * cfg.n_heads * nl * cfg.l_ctx * cfg.head_dim      # nl holds the batch
    total = sum(seg)
    return [v / total for v in seg]


def simulate_step(blocks, chunk_bytes, r, link_gbs, chunk_overhead_us=0.0, n_steps=4):
    """Steady-state step time of the two-stream schedule, chunk by chunk.

    blocks: one dict per block of the stack with 'blob_bytes', 't_comp_ms' and 'shares' (per-chunk
    compute shares).  Copy stream: the streamed chunks of block i+1 are copied in order once the
    prefetch has been issued (start of block i, Sec. 2.2), the chunks of block i are out and block
    i-1, the last tenant of the slot, has finished.  Compute stream: segment k of a block starts
    when segment k-1 has ended and, unless chunk k is resident (the first round(r*n_chunks) chunks,
    Sec. 3.3), when chunk k has landed.  Returns (step_ms, exposed_ms, weight_memory_bytes)."""
    L = len(blocks)
    ms_per_byte = 1e3 / (link_gbs * 1e9)
    info = []
    for b in blocks:
        n = -(-b["blob_bytes"] // chunk_bytes)
        n_res = int((r * n + 0.5) // 1)
        res_bytes = min(b["blob_bytes"], n_res * chunk_bytes)
        sizes = [min(chunk_bytes, b["blob_bytes"] - k * chunk_bytes) for k in range(n)]
        info.append((n, n_res, res_bytes, sizes))
    finish = {}            # block instance -> end of its compute
    landed = {}            # block instance -> landing time of each streamed chunk
    link_free = 0.0

    def copy(i, issued):
        nonlocal link_free
        n, n_res, _, sizes = info[i % L]
        t = max(link_free, issued, finish.get(i - 2, 0.0))
        times = {}
        for k in range(n_res, n):
            t += chunk_overhead_us * 1e-3 + sizes[k] * ms_per_byte
            times[k] = t
        landed[i] = times
        link_free = t

    copy(0, 0.0)
    total = n_steps * L
    for i in range(total):
        start = finish.get(i - 1, 0.0)
        if i + 1 < total:
            copy(i + 1, start)
        t = start
        b = blocks[i % L]
        for k, share in enumerate(b["shares"]):
            t = max(t, landed[i].get(k, 0.0)) + share * b["t_comp_ms"]
        finish[i] = t
    step = finish[total - 1] - finish[total - 1 - L]
    compute = sum(b["t_comp_ms"] for b in blocks)
    slot = max(b["blob_bytes"] - inf[2] for b, inf in zip(blocks, info))
    memory = sum(inf[2] for inf in info) + 2 * slot
    return step, step - compute, memory
