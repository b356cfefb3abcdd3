"""ctypes binding of libchunkflow.so: argument marshalling only.

Every step of the block path runs in the HIP library; PyTorch is used for device memory,
pinned host memory and stream handles.  Loading fails loudly when the library has not been
built (`python paper_2605_11335_amd/build.py`): there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libchunkflow.so")

CF_SINGLE_STREAM, CF_DIT_CROSS, CF_DOUBLE_STREAM = 0, 1, 2
CF_OK, CF_ERR_ARG, CF_ERR_STATE, CF_ERR_HIP, CF_ERR_NOMEM, CF_ERR_UNSUPPORTED = 0, -1, -2, -3, -4, -5


class cf_model_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_blocks", C.c_int32), ("d", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("f", C.c_int32), ("n_total", C.c_int32), ("sp_degree", C.c_int32),
                ("sp_rank", C.c_int32), ("n_txt_total", C.c_int32), ("l_ctx", C.c_int32),
                ("qk_rmsnorm", C.c_int32), ("gelu_erf", C.c_int32), ("batch", C.c_int32), ("chunk_bytes", C.c_uint64)]


class cf_tensor_slot(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("offset", C.c_uint64), ("rows", C.c_uint32), ("cols", C.c_uint32)]


class cf_block_io(C.Structure):
    _fields_ = [("x", C.c_void_p), ("x_txt", C.c_void_p), ("temb", C.c_void_p), ("ctx", C.c_void_p),
                ("peer_q", C.c_void_p), ("peer_k", C.c_void_p), ("peer_v", C.c_void_p), ("peer_attn", C.c_void_p),
                ("rope_cos", C.c_void_p), ("rope_sin", C.c_void_p),
                ("y", C.c_void_p), ("y_txt", C.c_void_p),
                ("send_q", C.c_void_p), ("send_k", C.c_void_p), ("send_v", C.c_void_p), ("send_attn", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_uint64),
                ("x_sample_stride", C.c_int64), ("x_txt_sample_stride", C.c_int64)]


class cf_stats_t(C.Structure):
    _fields_ = [("h2d_bytes", C.c_uint64), ("h2d_chunks", C.c_uint64), ("resident_bytes", C.c_uint64),
                ("blob_bytes", C.c_uint64), ("weight_memory_bytes", C.c_uint64),
                ("comm_bytes_h2d", C.c_uint64), ("comm_bytes_d2h", C.c_uint64), ("pauses", C.c_uint64),
                ("model_resident_bytes", C.c_uint64), ("model_blob_bytes", C.c_uint64),
                ("blocks_one_wait", C.c_uint64)]


class cf_kernel_time(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("launches", C.c_uint64), ("total_ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double)]


class cf_machine_t(C.Structure):
    _fields_ = [("t_comp_ms", C.c_double * 3), ("link_gbs", C.c_double), ("chunk_overhead_us", C.c_double)]


class cf_sim_result(C.Structure):
    _fields_ = [("step_ms", C.c_double), ("compute_ms", C.c_double), ("exposed_ms", C.c_double),
                ("weight_memory_bytes", C.c_uint64), ("h2d_bytes_per_step", C.c_uint64),
                ("resident_fraction", C.c_double)]


class cf_tune_choice(C.Structure):
    _fields_ = [("chunk_bytes", C.c_uint64), ("r", C.c_double), ("feasible", C.c_int32), ("sim", cf_sim_result)]


#: what include/chunkflow.h declares: the block path's contract
CORE_EXPORTS = ["cf_create", "cf_destroy", "cf_last_error", "cf_blob_bytes", "cf_n_chunks", "cf_blob_layout",
                "cf_set_block_kinds", "cf_block_kind_of", "cf_blob_bytes_of", "cf_n_chunks_of", "cf_blob_layout_of",
                "cf_workspace_bytes", "cf_plan_panels", "cf_simulate", "cf_tune", "cf_register_block",
                "set_resident_fraction", "chunked_prefetch_begin", "chunked_prefetch_wait", "dit_block_fwd",
                "cf_set_contention", "cf_comm_begin", "cf_comm_end", "cf_checksum_block", "cf_read_block", "cf_stats",
                "cf_stats_reset", "cf_set_profiling", "cf_set_adaptive_waits", "cf_kernel_times", "cf_kernel_times_reset",
                "cf_sync", "cf_op_checksum", "cf_op_checksum_noalloc"]
#: what include/chunkflow_diag.h declares: single-kernel hooks, planner views, the matrix-core rate probe
DIAG_EXPORTS = ["cf_plan_attention", "cf_plan_linear", "cf_op_linear", "cf_op_linear_residual", "cf_op_attention",
                "cf_op_ln_modulate", "cf_op_modvec", "cf_op_mfma_rate", "cf_op_mix_rate"]
EXPORTS = CORE_EXPORTS + DIAG_EXPORTS

_lib = None


class ChunkflowError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"chunkflow error {code}: {msg}")
        self.code = code


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2605_11335_amd/build.py` "
                              "(there is no CPU or PyTorch fallback for the block path)")
        # PyTorch ships its own HIP runtime; load it first so that this library binds to the same
        # one (two runtimes in one process do not share the device)
        import torch  # noqa: F401
        _lib = C.CDLL(LIB_PATH)
        _lib.cf_last_error.restype = C.c_char_p
        _lib.cf_last_error.argtypes = [C.c_void_p]
        for name in EXPORTS:
            fn = getattr(_lib, name)
            if name != "cf_last_error":
                fn.restype = C.c_int
        _lib.set_resident_fraction.argtypes = [C.c_void_p, C.c_double, C.POINTER(C.c_double)]
        _lib.cf_set_contention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64, C.c_int32]
        _lib.cf_set_adaptive_waits.argtypes = [C.c_void_p, C.c_int32]
        _lib.cf_plan_panels.argtypes = [C.c_void_p, C.c_char_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.POINTER(C.c_int32)]
        _lib.cf_plan_attention.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
        _lib.cf_plan_linear.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
        _lib.cf_register_block.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_uint64]
        _lib.cf_set_block_kinds.argtypes = [C.c_void_p, C.c_void_p, C.c_int32]
        _lib.cf_simulate.argtypes = [C.c_void_p, C.c_double, C.POINTER(cf_machine_t), C.POINTER(cf_sim_result)]
        _lib.cf_tune.argtypes = [C.c_void_p, C.POINTER(cf_machine_t), C.c_void_p, C.c_int32, C.c_int32, C.c_uint64,
                                 C.c_double, C.POINTER(cf_tune_choice)]
        _lib.cf_block_kind_of.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        _lib.cf_blob_bytes_of.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        _lib.cf_n_chunks_of.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        _lib.cf_blob_layout_of.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        _lib.chunked_prefetch_begin.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        _lib.chunked_prefetch_wait.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        _lib.dit_block_fwd.argtypes = [C.c_void_p, C.c_int32, C.POINTER(cf_block_io), C.c_void_p]
        _lib.cf_checksum_block.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        _lib.cf_read_block.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        _lib.cf_comm_begin.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.cf_comm_end.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.cf_op_linear.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_uint64, C.c_int64, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_int32, C.c_int32, C.c_void_p]
        _lib.cf_op_linear_residual.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_uint64, C.c_int64, C.c_int32,
                                               C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.cf_op_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                         C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        _lib.cf_op_ln_modulate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        _lib.cf_op_modvec.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        _lib.cf_op_mfma_rate.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        _lib.cf_op_mix_rate.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        _lib.cf_op_checksum.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p]
        _lib.cf_op_checksum_noalloc.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p]
    return _lib


def _check(rc: int, ctx=None):
    if rc != 0:
        msg = lib().cf_last_error(ctx) or b""
        raise ChunkflowError(rc, msg.decode(errors="replace"))


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    return t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        return None
    return stream.cuda_stream


def desc_from_config(cfg, chunk_bytes: int) -> cf_model_desc:
    return cf_model_desc(kind=cfg.kind, n_blocks=cfg.n_blocks, d=cfg.d, n_heads=cfg.n_heads, head_dim=cfg.head_dim,
                         f=cfg.f, n_total=cfg.n_total, sp_degree=cfg.sp_degree, sp_rank=cfg.sp_rank,
                         n_txt_total=cfg.n_txt, l_ctx=cfg.l_ctx, qk_rmsnorm=int(cfg.qk_rmsnorm),
                         gelu_erf=int(cfg.gelu_erf), batch=int(getattr(cfg, "batch", 1)), chunk_bytes=chunk_bytes)


class Context:
    """Owns one cf_ctx.  Method names are the C entry points'."""

    def __init__(self, desc: cf_model_desc):
        self._h = C.c_void_p()
        rc = lib().cf_create(C.byref(desc), C.byref(self._h))
        if rc != 0:
            raise ChunkflowError(rc, (lib().cf_last_error(None) or b"").decode())
        self.desc = desc
        self._keep = []          # pinned blobs must outlive the context

    def close(self):
        if self._h:
            lib().cf_destroy(self._h)
            self._h = C.c_void_p()
            self._keep.clear()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- layout
    def cf_set_block_kinds(self, kinds) -> None:
        arr = (C.c_int32 * len(kinds))(*[int(k) for k in kinds])
        _check(lib().cf_set_block_kinds(self._h, arr, len(kinds)), self._h)

    def cf_block_kind_of(self, block: int) -> int:
        v = C.c_int32()
        _check(lib().cf_block_kind_of(self._h, block, C.byref(v)), self._h)
        return v.value

    def cf_blob_bytes(self, block: int = 0) -> int:
        v = C.c_uint64()
        _check(lib().cf_blob_bytes_of(self._h, block, C.byref(v)), self._h)
        return v.value

    def cf_n_chunks(self, block: int = 0) -> int:
        v = C.c_int32()
        _check(lib().cf_n_chunks_of(self._h, block, C.byref(v)), self._h)
        return v.value

    def cf_workspace_bytes(self) -> int:
        v = C.c_uint64()
        _check(lib().cf_workspace_bytes(self._h, C.byref(v)), self._h)
        return v.value

    def cf_plan_panels(self, tensor: str, m_rows: int, n_resident_chunks: int) -> List[tuple]:
        n = C.c_int32(0)
        _check(lib().cf_plan_panels(self._h, tensor.encode(), m_rows, n_resident_chunks, None, None, None, C.byref(n)), self._h)
        r0, r1, w = (C.c_int32 * n.value)(), (C.c_int32 * n.value)(), (C.c_int32 * n.value)()
        _check(lib().cf_plan_panels(self._h, tensor.encode(), m_rows, n_resident_chunks, r0, r1, w, C.byref(n)), self._h)
        return [(r0[i], r1[i], w[i]) for i in range(n.value)]

    # ---- overlap model
    @staticmethod
    def _machine(t_comp_ms, link_gbs: float, chunk_overhead_us: float = 0.0) -> cf_machine_t:
        """t_comp_ms: per-block compute time, one number or {kind: ms}."""
        t = [float(t_comp_ms)] * 3 if not isinstance(t_comp_ms, dict) else [float(t_comp_ms.get(k, 0.0)) for k in range(3)]
        return cf_machine_t((C.c_double * 3)(*t), link_gbs, chunk_overhead_us)

    @staticmethod
    def _sim_dict(s: cf_sim_result) -> dict:
        return {n: getattr(s, n) for n, _ in cf_sim_result._fields_}

    def cf_simulate(self, r: float, t_comp_ms, link_gbs: float, chunk_overhead_us: float = 0.0) -> dict:
        out = cf_sim_result()
        m = self._machine(t_comp_ms, link_gbs, chunk_overhead_us)
        _check(lib().cf_simulate(self._h, r, C.byref(m), C.byref(out)), self._h)
        return self._sim_dict(out)

    def cf_tune(self, t_comp_ms, link_gbs: float, chunk_candidates, r_steps: int, memory_budget_bytes: int = 0,
                step_target_ms: float = 0.0, chunk_overhead_us: float = 0.0) -> dict:
        out = cf_tune_choice()
        m = self._machine(t_comp_ms, link_gbs, chunk_overhead_us)
        cand = (C.c_uint64 * len(chunk_candidates))(*[int(v) for v in chunk_candidates])
        _check(lib().cf_tune(self._h, C.byref(m), cand, len(chunk_candidates), r_steps, memory_budget_bytes,
                             step_target_ms, C.byref(out)), self._h)
        return dict(chunk_bytes=out.chunk_bytes, r=out.r, feasible=bool(out.feasible), **self._sim_dict(out.sim))

    def cf_blob_layout(self, block: int = 0) -> List[dict]:
        n = C.c_int32(0)
        _check(lib().cf_blob_layout_of(self._h, block, None, C.byref(n)), self._h)
        arr = (cf_tensor_slot * n.value)()
        _check(lib().cf_blob_layout_of(self._h, block, arr, C.byref(n)), self._h)
        return [dict(name=a.name.decode(), offset=a.offset, rows=a.rows, cols=a.cols) for a in arr]

    def pack_blob(self, params: Dict[str, np.ndarray], out: np.ndarray, block: int = 0) -> None:
        """Place named bf16 tensors (uint16 bit patterns) at the library's offsets; pad is zero."""
        assert out.dtype == np.uint8 and out.size == self.cf_blob_bytes(block)
        out[:] = 0
        for t in self.cf_blob_layout(block):
            a = np.ascontiguousarray(params[t["name"]], dtype=np.uint16).reshape(-1)
            assert a.size == t["rows"] * t["cols"], t["name"]
            out[t["offset"]:t["offset"] + 2 * a.size] = a.view(np.uint8)

    # ---- weights
    def cf_register_block(self, block: int, pinned_blob) -> None:
        """pinned_blob: torch uint8 tensor allocated with pin_memory=True (kept alive here)."""
        self._keep.append(pinned_blob)
        _check(lib().cf_register_block(self._h, block, pinned_blob.data_ptr(), pinned_blob.numel()), self._h)

    def set_resident_fraction(self, r: float) -> float:
        actual = C.c_double()
        _check(lib().set_resident_fraction(self._h, float(r), C.byref(actual)), self._h)
        return actual.value

    def chunked_prefetch_begin(self, block: int, copy_stream) -> None:
        _check(lib().chunked_prefetch_begin(self._h, block, _stream_handle(copy_stream)), self._h)

    def chunked_prefetch_wait(self, block: int, chunk: int, compute_stream) -> None:
        _check(lib().chunked_prefetch_wait(self._h, block, chunk, _stream_handle(compute_stream)), self._h)

    def dit_block_fwd(self, block: int, io: cf_block_io, compute_stream) -> None:
        _check(lib().dit_block_fwd(self._h, block, C.byref(io), _stream_handle(compute_stream)), self._h)

    def cf_set_contention(self, comm_stream, host_pinned, bytes_per_collective: int, pause_resume) -> None:
        """pause_resume: 0 / False = off, 1 / True = one chunk in flight, 2 = two."""
        if host_pinned is not None:
            self._keep.append(host_pinned)
        _check(lib().cf_set_contention(self._h, _stream_handle(comm_stream), _ptr(host_pinned),
                                       0 if host_pinned is None else host_pinned.numel(),
                                       bytes_per_collective, int(pause_resume)), self._h)

    def cf_comm_begin(self, comm_stream, compute_stream) -> None:
        _check(lib().cf_comm_begin(self._h, _stream_handle(comm_stream), _stream_handle(compute_stream)), self._h)

    def cf_comm_end(self, comm_stream, compute_stream) -> None:
        _check(lib().cf_comm_end(self._h, _stream_handle(comm_stream), _stream_handle(compute_stream)), self._h)

    def cf_checksum_block(self, block: int, stream=None) -> List[int]:
        out = (C.c_uint64 * self.cf_n_chunks(block))()
        _check(lib().cf_checksum_block(self._h, block, out, _stream_handle(stream)), self._h)
        return list(out)

    def cf_read_block(self, block: int, stream=None) -> np.ndarray:
        out = np.empty(self.cf_blob_bytes(block), dtype=np.uint8)
        _check(lib().cf_read_block(self._h, block, out.ctypes.data, _stream_handle(stream)), self._h)
        return out

    def cf_stats(self) -> dict:
        s = cf_stats_t()
        _check(lib().cf_stats(self._h, C.byref(s)), self._h)
        return {k: getattr(s, k) for k, _ in cf_stats_t._fields_}

    def cf_stats_reset(self) -> None:
        _check(lib().cf_stats_reset(self._h), self._h)

    def cf_set_profiling(self, on: bool) -> None:
        _check(lib().cf_set_profiling(self._h, int(on)), self._h)

    def cf_set_adaptive_waits(self, on: bool) -> None:
        _check(lib().cf_set_adaptive_waits(self._h, int(on)), self._h)

    def cf_kernel_times(self) -> List[dict]:
        n = C.c_int32(64)
        arr = (cf_kernel_time * 64)()
        _check(lib().cf_kernel_times(self._h, arr, C.byref(n)), self._h)
        return [dict(name=arr[i].name.decode(), launches=arr[i].launches, total_ms=arr[i].total_ms,
                     flops=arr[i].flops, bytes=arr[i].bytes) for i in range(n.value)]

    def cf_kernel_times_reset(self) -> None:
        _check(lib().cf_kernel_times_reset(self._h), self._h)

    def cf_sync(self) -> None:
        _check(lib().cf_sync(self._h), self._h)


def make_io(**tensors) -> cf_block_io:
    """cf_block_io from torch device tensors (by field name); `workspace` is a uint8 tensor;
    x_sample_stride / x_txt_sample_stride are plain integers."""
    io = cf_block_io()
    for k, t in tensors.items():
        if t is None:
            continue
        if k.endswith("_sample_stride"):
            setattr(io, k, int(t))
            continue
        setattr(io, k, t.data_ptr())
        if k == "workspace":
            io.workspace_bytes = t.numel() * t.element_size()
    return io


# ---- single kernels (device tensors are torch tensors; bf16 data as torch.bfloat16 or int16 views)
def cf_op_linear(A, blob, w_off, bias_off, M, N, K, out0, out1=None, n_split=None, n0=0, n1=None, lda=None,
                 ld0=None, ld1=None, gelu_erf=False, stream=None):
    n1 = N if n1 is None else n1
    n_split = N if n_split is None else n_split
    _check(lib().cf_op_linear(_ptr(A), K if lda is None else lda, _ptr(blob), w_off, bias_off, M, N, K, n0, n1, n_split,
                              _ptr(out0), (n_split if ld0 is None else ld0), _ptr(out1),
                              ((N - n_split) if ld1 is None else ld1), int(gelu_erf), _stream_handle(stream)))


def cf_plan_attention(H: int, nq: int, nk: int, head_dim: int) -> int:
    """Waves per workgroup an attention launch of this shape takes (host arithmetic only)."""
    out = C.c_int32()
    _check(lib().cf_plan_attention(H, nq, nk, head_dim, C.byref(out)))
    return out.value


def cf_plan_linear(m_rows: int, n_features: int) -> int:
    """Tile height (256 or 128) a linear layer of this shape is launched with (host arithmetic only)."""
    out = C.c_int32()
    _check(lib().cf_plan_linear(m_rows, n_features, C.byref(out)))
    return out.value


def cf_op_mfma_rate(iters: int, random_operands: bool, out, stream=None) -> None:
    _check(lib().cf_op_mfma_rate(iters, int(random_operands), _ptr(out), _stream_handle(stream)))


def cf_op_mix_rate(iters: int, waves: int, reads_per_16: int, valu_per_mfma: int, exp_per_mfma: int, out, stream=None) -> None:
    _check(lib().cf_op_mix_rate(iters, waves, reads_per_16, valu_per_mfma, exp_per_mfma, _ptr(out), _stream_handle(stream)))


def cf_op_linear_residual(A, blob, w_off, bias_off, M, N, K, resid, gate, y, lda=None, stream=None):
    _check(lib().cf_op_linear_residual(_ptr(A), K if lda is None else lda, _ptr(blob), w_off, bias_off, M, N, K,
                                       _ptr(resid), _ptr(gate), _ptr(y), _stream_handle(stream)))


def cf_op_attention(Q, K, Vt, O, H, nq, nk, nk_pad, hd, stream=None):
    _check(lib().cf_op_attention(_ptr(Q), _ptr(K), _ptr(Vt), _ptr(O), H, nq, nk, nk_pad, hd, _stream_handle(stream)))


def cf_op_ln_modulate(x, shift, scale, xn, rows, d, stream=None):
    _check(lib().cf_op_ln_modulate(_ptr(x), _ptr(shift), _ptr(scale), _ptr(xn), rows, d, _stream_handle(stream)))


def cf_op_modvec(blob, w_off, b_off, t, m, n, K, stream=None):
    _check(lib().cf_op_modvec(_ptr(blob), w_off, b_off, _ptr(t), _ptr(m), n, K, _stream_handle(stream)))


def cf_op_checksum(data, nbytes, first_word, stream=None) -> int:
    out = C.c_uint64()
    _check(lib().cf_op_checksum(_ptr(data), nbytes, first_word, C.byref(out), _stream_handle(stream)))
    return out.value


def cf_op_checksum_noalloc(data, nbytes, first_word, dev_out, stream=None) -> None:
    """Checksum of a device byte range into a device uint64 (torch int64 tensor of one element);
    enqueues only: the caller synchronises before reading dev_out."""
    _check(lib().cf_op_checksum_noalloc(_ptr(data), nbytes, first_word, _ptr(dev_out), _stream_handle(stream)))
