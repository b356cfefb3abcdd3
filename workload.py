"""Workload shapes and seeded synthetic tensors for the offloaded-DiT block path.

This module is data only: it names the benchmark configurations (shapes of one
GPU's Ulysses share of a DiT block) and draws every input tensor from a seeded
counter-based generator (NumPy's Philox).  It holds none of the method's
arithmetic -- no normalisation, no matmul, no softmax -- so that the CPU oracle
and the HIP path can both take their inputs from here without sharing any
compute code.  The only numeric operation is the storage-format conversion
float32 -> bfloat16 (round to nearest even), which defines what "a bf16 tensor
drawn from N(0, s)" means.

Tensors are returned either as ``uint16`` arrays holding bf16 bit patterns
(weights, peer activations) or as ``float32`` arrays whose values are exactly
bf16-representable (the residual stream ``x`` and the timestep embedding).
"""
from __future__ import annotations

import dataclasses
import zlib
from typing import Dict, List, Tuple

import numpy as np

BASE_SEED = 20260511

KIND_SINGLE = 0   # fused parallel attention+MLP block (MM-DiT single-stream, App. B)
KIND_DIT = 1      # self-attn, cross-attn to text, FFN (DiT block, App. B)
KIND_DOUBLE = 2   # separate img/txt weights, joint attention (MM-DiT double-stream, App. B)


@dataclasses.dataclass(frozen=True)
class BlockConfig:
    """Shape of one GPU's share of a stack of identical DiT blocks."""
    name: str
    kind: int
    n_blocks: int
    d: int              # hidden size
    n_heads: int        # H (global)
    head_dim: int       # hd
    f: int              # MLP width
    n_total: int        # N: full joint sequence the attention runs over
    sp_degree: int = 1  # P: Ulysses degree
    sp_rank: int = 0
    n_txt: int = 0      # double-stream: text tokens in the joint sequence (global)
    l_ctx: int = 0      # DiT block: cross-attention context length
    qk_rmsnorm: bool = True
    n_chunks: int = 8   # chunks per block the config asks for (chunk_bytes derived)
    temb_std: float = 1.0
    n_double: int = 0   # mixed model: the first n_double blocks are double-stream, the rest `kind`
    rope: bool = False  # hand rotary position tables to the block (q, k rotated after the norm)
    gelu_erf: bool = False  # MLP activation x * Phi(x) instead of its tanh approximation
    batch: int = 1      # B: independent samples per forward (own activations, timestep embedding, peers)

    @property
    def n_local(self) -> int:
        return self.n_total // self.sp_degree

    @property
    def h_local(self) -> int:
        return self.n_heads // self.sp_degree

    @property
    def n_txt_local(self) -> int:
        return self.n_txt // self.sp_degree

    def with_(self, **kw) -> "BlockConfig":
        return dataclasses.replace(self, **kw)

    def kind_of(self, block: int) -> int:
        return KIND_DOUBLE if block < self.n_double else self.kind

    @property
    def kinds(self) -> List[int]:
        return [self.kind_of(b) for b in range(self.n_blocks)]

    def block_cfg(self, block: int) -> "BlockConfig":
        """The configuration of one block of a (possibly mixed) stack, as a one-kind config."""
        return dataclasses.replace(self, kind=self.kind_of(block), n_double=0)


def _temb_std(d: int) -> float:
    # The toy configuration draws the timestep embedding from N(0,1) at d=512, which
    # gives shift/scale/gate a standard deviation of 0.02*sqrt(512) ~= 0.45.  Wider
    # models keep that modulation scale (a trained adaLN emits O(0.1-1) values), so
    # the embedding's standard deviation shrinks with sqrt(512/d).
    return float(np.sqrt(512.0 / d)) if d > 512 else 1.0


CONFIGS: Dict[str, BlockConfig] = {
    # C1: toy, all heads local.
    "toy": BlockConfig("toy", KIND_SINGLE, n_blocks=2, d=512, n_heads=8, head_dim=64, f=2048,
                       n_total=512, sp_degree=1, qk_rmsnorm=False, n_chunks=4, temb_std=1.0),
    # C2: Flux-like single-stream share (512 text + 4096 image tokens, P=2).
    "flux": BlockConfig("flux", KIND_SINGLE, n_blocks=8, d=3072, n_heads=24, head_dim=128, f=12288,
                        n_total=4608, sp_degree=2, qk_rmsnorm=True, n_chunks=8,
                        temb_std=_temb_std(3072)),
    # C3: Wan-5B-like DiT block share (31x22x40 latent grid, 512 text tokens).
    "wan": BlockConfig("wan", KIND_DIT, n_blocks=30, d=3072, n_heads=24, head_dim=128, f=14336,
                       n_total=27280, sp_degree=2, l_ctx=512, qk_rmsnorm=True, n_chunks=8,
                       temb_std=_temb_std(3072)),
    # C4: HunyuanVideo-13B-like double-stream share (33x45x80 grid + 256 text tokens).
    "hunyuan": BlockConfig("hunyuan", KIND_DOUBLE, n_blocks=20, d=3072, n_heads=24, head_dim=128,
                           f=12288, n_total=118800 + 256, sp_degree=2, n_txt=256, qk_rmsnorm=True,
                           n_chunks=8, temb_std=_temb_std(3072)),
    # The MMDiT composition of a Flux-like denoiser (App. B): 19 double-stream blocks, then 38
    # single-stream blocks over the concatenated 512 text + 4096 image tokens, P=2.
    "flux_mm": BlockConfig("flux_mm", KIND_SINGLE, n_blocks=57, d=3072, n_heads=24, head_dim=128, f=12288,
                           n_total=4608, sp_degree=2, n_txt=512, qk_rmsnorm=True, n_chunks=8,
                           temb_std=_temb_std(3072), n_double=19),
    # The composition of a HunyuanVideo-like denoiser (App. C, Table 1): 20 double-stream blocks,
    # then 40 single-stream blocks over the same 118800 video + 256 text tokens, P=2.
    "hunyuan_mm": BlockConfig("hunyuan_mm", KIND_SINGLE, n_blocks=60, d=3072, n_heads=24, head_dim=128, f=12288,
                              n_total=118800 + 256, sp_degree=2, n_txt=256, qk_rmsnorm=True, n_chunks=8,
                              temb_std=_temb_std(3072), n_double=20),
    # The same composition small enough for the CPU oracle in seconds.
    "toy_mm": BlockConfig("toy_mm", KIND_SINGLE, n_blocks=3, d=512, n_heads=8, head_dim=64, f=2048,
                          n_total=640, sp_degree=2, n_txt=128, qk_rmsnorm=True, n_chunks=4, temb_std=1.0,
                          n_double=1),
}


# --------------------------------------------------------------------------------------
# storage-format helpers
# --------------------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even. Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------------------
# seeded draws
# --------------------------------------------------------------------------------------

def _rng(cfg_name: str, block: int, tensor: str) -> np.random.Generator:
    key = zlib.crc32(f"{cfg_name}/{tensor}".encode())
    return np.random.Generator(np.random.Philox(key=[BASE_SEED, (block << 32) | key]))


def normal_bf16(cfg_name: str, block: int, tensor: str, shape, std: float, mean: float = 0.0) -> np.ndarray:
    """Seeded N(mean, std) tensor rounded to bf16, returned as uint16 bit patterns."""
    rng = _rng(cfg_name, block, tensor)
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for s in range(0, n, step):
        e = min(n, s + step)
        v = rng.standard_normal(e - s, dtype=np.float32)
        v *= np.float32(std)
        if mean != 0.0:
            v += np.float32(mean)
        out[s:e] = f32_to_bf16_bits(v)
    return out.reshape(shape)


def param_specs(cfg: BlockConfig) -> List[Tuple[str, Tuple[int, ...], float, float]]:
    """(name, shape, std, mean) of every weight tensor of one block, in the order the
    block consumes them.  Linear weights are [out_features, in_features]."""
    d, f, hd = cfg.d, cfg.f, cfg.head_dim
    w, one = 0.02, 1.0
    if cfg.kind == KIND_SINGLE:
        specs = [("b_mod", (3 * d,), w, 0.0), ("w_mod", (3 * d, d), w, 0.0),
                 ("b1", (3 * d + f,), w, 0.0)]
        if cfg.qk_rmsnorm:
            specs += [("q_norm", (hd,), w, one), ("k_norm", (hd,), w, one)]
        specs += [("w1", (3 * d + f, d), w, 0.0), ("b2", (d,), w, 0.0), ("w2", (d, d + f), w, 0.0)]
        return specs
    if cfg.kind == KIND_DIT:
        specs = [("b_mod", (6 * d,), w, 0.0), ("w_mod", (6 * d, d), w, 0.0),
                 ("b_qkv", (3 * d,), w, 0.0)]
        if cfg.qk_rmsnorm:
            specs += [("q_norm", (hd,), w, one), ("k_norm", (hd,), w, one)]
        specs += [("w_qkv", (3 * d, d), w, 0.0), ("b_o", (d,), w, 0.0), ("w_o", (d, d), w, 0.0),
                  ("ln_c_w", (d,), w, one), ("ln_c_b", (d,), w, 0.0),
                  ("b_cq", (d,), w, 0.0)]
        if cfg.qk_rmsnorm:
            specs += [("cq_norm", (hd,), w, one), ("ck_norm", (hd,), w, one)]
        specs += [("w_cq", (d, d), w, 0.0), ("b_ckv", (2 * d,), w, 0.0), ("w_ckv", (2 * d, d), w, 0.0),
                  ("b_co", (d,), w, 0.0), ("w_co", (d, d), w, 0.0),
                  ("b_up", (f,), w, 0.0), ("w_up", (f, d), w, 0.0),
                  ("b_down", (d,), w, 0.0), ("w_down", (d, f), w, 0.0)]
        return specs
    if cfg.kind == KIND_DOUBLE:
        specs = []
        for s in ("img", "txt"):
            specs += [(f"{s}_b_mod", (6 * d,), w, 0.0), (f"{s}_w_mod", (6 * d, d), w, 0.0)]
        for s in ("img", "txt"):
            specs += [(f"{s}_b_qkv", (3 * d,), w, 0.0)]
            if cfg.qk_rmsnorm:
                specs += [(f"{s}_q_norm", (hd,), w, one), (f"{s}_k_norm", (hd,), w, one)]
            specs += [(f"{s}_w_qkv", (3 * d, d), w, 0.0)]
        for s in ("img", "txt"):
            specs += [(f"{s}_b_o", (d,), w, 0.0), (f"{s}_w_o", (d, d), w, 0.0)]
        for s in ("img", "txt"):
            specs += [(f"{s}_b_up", (f,), w, 0.0), (f"{s}_w_up", (f, d), w, 0.0),
                      (f"{s}_b_down", (d,), w, 0.0), (f"{s}_w_down", (d, f), w, 0.0)]
        return specs
    raise ValueError(f"unknown block kind {cfg.kind}")


def gen_block_params(cfg: BlockConfig, block: int) -> Dict[str, np.ndarray]:
    """All weight tensors of one block as bf16 bit patterns (uint16), distinct per block."""
    return {name: normal_bf16(cfg.name, block, name, shape, std, mean)
            for name, shape, std, mean in param_specs(cfg)}


def gen_block_inputs(cfg: BlockConfig, block: int, sample: int = None) -> Dict[str, np.ndarray]:
    """Activations entering one block on this rank, plus the seeded stand-ins for what the
    Ulysses all-to-alls would have delivered from the other ranks.

    x, temb, (x_txt), (ctx): float32 arrays with bf16-representable values.
    peer_q/k/v: [h_local, n_total - n_local, head_dim] bf16 bits (q,k unit-variance like
    RMS-normalised projections; v half that).  peer_attn: [n_local, H - h_local, head_dim].

    With cfg.batch > 1 and no `sample`, every array but the rotary tables is the stack of the
    samples' arrays along a new leading axis; `sample` = b gives sample b alone (sample 0 of a
    batch is the batch-1 input).
    """
    if sample is None and cfg.batch > 1:
        per = [gen_block_inputs(cfg, block, b) for b in range(cfg.batch)]
        return {k: (per[0][k] if k.startswith("rope_") else np.stack([p[k] for p in per])) for k in per[0]}
    d, hd = cfg.d, cfg.head_dim
    nl, hl = cfg.n_local, cfg.h_local
    nrem = cfg.n_total - nl
    out: Dict[str, np.ndarray] = {}
    tag = lambda t: t if not sample else f"{t}#{sample}"
    act = lambda t, shape, std=1.0: bf16_bits_to_f32(normal_bf16(cfg.name, block, tag(t), shape, std))
    if cfg.kind == KIND_DOUBLE:
        tl = cfg.n_txt_local
        out["x"] = act("x", (nl - tl, d))
        out["x_txt"] = act("x_txt", (tl, d))
    else:
        out["x"] = act("x", (nl, d))
    out["temb"] = act("temb", (d,), cfg.temb_std)
    if cfg.kind == KIND_DIT:
        out["ctx"] = act("ctx", (cfg.l_ctx, d))
    if cfg.rope:
        # seeded angles, one per (local row, pair of head dimensions), the same for every head and sample
        ang = _rng(cfg.name, block, "rope").uniform(0.0, 2.0 * np.pi, size=(nl, hd // 2))
        out["rope_cos"] = np.cos(ang).astype(np.float32)
        out["rope_sin"] = np.sin(ang).astype(np.float32)
    if cfg.sp_degree > 1:
        out["peer_q"] = normal_bf16(cfg.name, block, tag("peer_q"), (hl, nrem, hd), 1.0)
        out["peer_k"] = normal_bf16(cfg.name, block, tag("peer_k"), (hl, nrem, hd), 1.0)
        out["peer_v"] = normal_bf16(cfg.name, block, tag("peer_v"), (hl, nrem, hd), 0.5)
        out["peer_attn"] = normal_bf16(cfg.name, block, tag("peer_attn"), (nl, cfg.n_heads - hl, hd), 0.5)
    return out


def local_positions(cfg: BlockConfig) -> np.ndarray:
    """Positions, in the joint N-token sequence, of this rank's local tokens (ascending).
    Tokens split contiguously per stream: text rows first (when the joint sequence has any), then
    image rows."""
    r, p = cfg.sp_rank, cfg.sp_degree
    if cfg.n_txt > 0:
        tl = cfg.n_txt_local
        il = cfg.n_local - tl
        txt = np.arange(r * tl, (r + 1) * tl)
        img = cfg.n_txt + np.arange(r * il, (r + 1) * il)
        return np.concatenate([txt, img])
    return np.arange(r * cfg.n_local, (r + 1) * cfg.n_local)


def remote_positions(cfg: BlockConfig) -> np.ndarray:
    mask = np.ones(cfg.n_total, dtype=bool)
    mask[local_positions(cfg)] = False
    return np.nonzero(mask)[0]
