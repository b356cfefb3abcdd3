"""Drives the C entry points for a stack of blocks: pinned host blobs, device I/O tensors,
the three streams, and the per-step call sequence

    chunked_prefetch_begin(l+1)  ->  dit_block_fwd(l)        (Sec. 2.2, prefetch issued first)

Nothing here computes: tensors are allocated with PyTorch and handed to the library.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

from . import binding as B


def make_context(cfg, chunk_bytes: int) -> B.Context:
    """Context for a stack of blocks; a mixed stack (cfg.n_double leading double-stream blocks)
    gets its per-block kinds."""
    ctx = B.Context(B.desc_from_config(cfg, chunk_bytes))
    if cfg.n_double:
        ctx.cf_set_block_kinds(cfg.kinds)
    return ctx


def blob_bytes_for(cfg) -> int:
    """Blob size of a block (the smallest over the kinds of a mixed stack)."""
    ctx = make_context(cfg, 1 << 20)
    n = min(ctx.cf_blob_bytes(b) for b in range(cfg.n_blocks))
    ctx.close()
    return n


def chunk_bytes_for(cfg, n_chunks: Optional[int] = None) -> int:
    """Chunk size that cuts the (smallest) blob into the configuration's number of chunks."""
    n_chunks = n_chunks or cfg.n_chunks
    blob = blob_bytes_for(cfg)
    return (blob + n_chunks - 1) // n_chunks // 256 * 256 + (256 if ((blob + n_chunks - 1) // n_chunks) % 256 else 0)


def _dev_bf16(bits: np.ndarray, device) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)


_STREAMS: Dict[str, tuple] = {}


def process_streams(device) -> tuple:
    """The process's (compute, copy, comm) streams on `device`, created once, back to back.  HIP
    multiplexes streams onto a few hardware queues (4 by default) in creation order, and two streams
    that share a queue run one after the other: a copy stream on the compute stream's queue hides
    behind nothing, a collective stream on the copy stream's queue waits for every enqueued chunk.
    Three streams created in a row sit on three different queues; triples created later in a process
    that has made many streams may not, so every runner of a process uses the same triple."""
    key = str(device)
    if key not in _STREAMS:
        _STREAMS[key] = tuple(torch.cuda.Stream(device=device) for _ in range(3))
    return _STREAMS[key]


class BlockRunner:
    def __init__(self, cfg, chunk_bytes: Optional[int] = None, device: str = "cuda:0", n_blocks: Optional[int] = None,
                 streams=None):
        """streams: (compute, copy, comm) torch streams to use instead of the process's triple."""
        self.cfg = cfg if n_blocks is None else cfg.with_(n_blocks=n_blocks)
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.chunk_bytes = chunk_bytes or chunk_bytes_for(self.cfg)
        self.ctx = make_context(self.cfg, self.chunk_bytes)
        self.blob_bytes_of = [self.ctx.cf_blob_bytes(b) for b in range(self.cfg.n_blocks)]
        self.total_blob_bytes = sum(self.blob_bytes_of)
        self.blob_bytes = self.blob_bytes_of[0]
        self.n_chunks = self.ctx.cf_n_chunks()
        self.compute, self.copy, self.comm = streams or process_streams(self.device)
        self.workspace = torch.empty(self.ctx.cf_workspace_bytes() + 256, dtype=torch.uint8, device=self.device)
        self.blobs: List[torch.Tensor] = []
        self.io_tensors: List[Dict[str, torch.Tensor]] = []
        self.ios: List[B.cf_block_io] = []

    # ---- weights
    def register_params(self, block: int, params: Dict[str, np.ndarray]) -> torch.Tensor:
        blob = torch.empty(self.blob_bytes_of[block], dtype=torch.uint8, pin_memory=True)
        self.ctx.pack_blob(params, blob.numpy(), block)
        self.ctx.cf_register_block(block, blob)
        while len(self.blobs) <= block:
            self.blobs.append(None)
        self.blobs[block] = blob
        return blob

    def register_blob(self, block: int, blob: torch.Tensor) -> None:
        """Register an already packed pinned blob (several blocks of one kind may share one: what
        travels over the link and what stays resident is per block either way)."""
        self.ctx.cf_register_block(block, blob)
        while len(self.blobs) <= block:
            self.blobs.append(None)
        self.blobs[block] = blob

    # ---- activations
    def make_io(self, inputs: Dict[str, np.ndarray]) -> Dict[str, torch.Tensor]:
        cfg, dev = self.cfg, self.device
        t: Dict[str, torch.Tensor] = {}
        f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
        t["x"] = f32(inputs["x"])
        t["temb"] = f32(inputs["temb"])
        t["y"] = torch.empty_like(t["x"])
        if "x_txt" in inputs:
            t["x_txt"] = f32(inputs["x_txt"])
            t["y_txt"] = torch.empty_like(t["x_txt"])
        for k in ("rope_cos", "rope_sin"):
            if k in inputs:
                t[k] = f32(inputs[k])
        if "ctx" in inputs:
            # context is handed over in bf16 (its values are bf16-representable already: exact)
            t["ctx"] = f32(inputs["ctx"]).to(torch.bfloat16)
        if cfg.sp_degree > 1:
            for k in ("peer_q", "peer_k", "peer_v", "peer_attn"):
                t[k] = _dev_bf16(inputs[k], dev)
            hl, ho, hd = cfg.h_local, cfg.n_heads - cfg.h_local, cfg.head_dim
            nl, nrem = cfg.n_local, cfg.n_total - cfg.n_local
            lead = (cfg.batch,) if cfg.batch > 1 else ()
            for k in ("send_q", "send_k", "send_v"):
                t[k] = torch.zeros(lead + (ho, nl, hd), dtype=torch.int16, device=dev)
            t["send_attn"] = torch.zeros(lead + (hl, nrem, hd), dtype=torch.int16, device=dev)
        # the tensors were produced on torch's current stream; the library reads and writes them on
        # streams of its own, so their producers must have finished first
        torch.cuda.current_stream(dev).synchronize()
        return t

    def io_struct(self, t: Dict[str, torch.Tensor]) -> B.cf_block_io:
        ws = self.workspace
        off = (-ws.data_ptr()) % 256
        io = B.make_io(**t)
        io.workspace = ws.data_ptr() + off
        io.workspace_bytes = ws.numel() - off
        return io

    # ---- execution
    def begin(self, block: int) -> None:
        self.ctx.chunked_prefetch_begin(block, self.copy)

    def fwd(self, block: int, io: B.cf_block_io) -> None:
        self.ctx.dit_block_fwd(block, io, self.compute)

    def run_block(self, block: int, tensors: Dict[str, torch.Tensor]) -> None:
        """One block in isolation: prefetch it, run it, wait."""
        self.begin(block)
        self.fwd(block, self.io_struct(tensors))
        self.ctx.cf_sync()

    def step(self, ios: List[B.cf_block_io], first_begun: bool = True) -> None:
        """One denoising step over all blocks, steady state: block 0's prefetch was issued during
        the previous step's last block (or by the caller), and the last block issues block 0's."""
        L = self.cfg.n_blocks
        if not first_begun:
            self.begin(0)
        for l in range(L):
            if L > 1:
                self.begin((l + 1) % L)
            self.fwd(l, ios[l])
            if L == 1:
                self.begin(0)

    def close(self):
        self.ctx.cf_sync()
        self.ctx.close()


def bits_of(t: torch.Tensor) -> np.ndarray:
    """int16 device tensor holding bf16 bit patterns -> uint16 numpy."""
    return t.cpu().numpy().view(np.uint16)
