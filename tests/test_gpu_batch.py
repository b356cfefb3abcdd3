"""Batches (B of App. B): B independent samples go through one block forward, the linear layers
on all B * n_local rows at once, attention per sample, the weights fetched once.  Every sample is
compared with the oracle run on that sample alone, and -- because every output element sees the
same k-order wherever its row sits -- with the library's own single-sample result bit for bit."""
import sys

import numpy as np
import pytest
import torch

import workload as wl
from oracle import block as ob
from paper_2605_11335_amd import binding as B
from paper_2605_11335_amd.runner import BlockRunner
from tests.util import bits_to_f64, max_abs, rel_l2

pytestmark = pytest.mark.gpu
REL_L2_TOL, MAX_ABS_TOL = 1e-2, 5e-2


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def close_to(got, want, what):
    r, m = rel_l2(got, want), max_abs(got, want)
    say(f"   {what}: rel_l2={r:.3e} max_abs={m:.3e}")
    assert r <= REL_L2_TOL and m <= MAX_ABS_TOL, what


def single_sample_outputs(cfg1, params, inputs_b, r):
    run = BlockRunner(cfg1, n_blocks=1)
    try:
        run.ctx.set_resident_fraction(r)
        run.register_params(0, params)
        t = run.make_io(inputs_b)
        run.run_block(0, t)
        return {k: v.cpu().numpy() for k, v in t.items() if k in ("y", "y_txt", "send_q", "send_k", "send_v", "send_attn")}
    finally:
        run.close()


def batch_vs_oracle_and_single(cfg, r=0.0):
    """cfg: one block, batch > 1."""
    cfg1 = cfg.with_(batch=1)
    params = wl.gen_block_params(cfg, 0)
    inputs = wl.gen_block_inputs(cfg, 0)
    run = BlockRunner(cfg, n_blocks=1)
    try:
        run.ctx.set_resident_fraction(r)
        run.register_params(0, params)
        t = run.make_io(inputs)
        assert t["x"].shape[0] == cfg.batch and t["temb"].shape == (cfg.batch, cfg.d)
        say(f"[{cfg.name}] batch {cfg.batch} kind {cfg.kind} P={cfg.sp_degree} r={r}")
        run.run_block(0, t)
        got = {k: v.cpu().numpy() for k, v in t.items() if v.dtype != torch.bfloat16}
    finally:
        run.close()
    for b in range(cfg.batch):
        inputs_b = wl.gen_block_inputs(cfg, 0, sample=b)
        for k in inputs_b:
            if not k.startswith("rope_"):
                assert np.array_equal(inputs_b[k], inputs[k][b])
        ref = ob.block_forward(cfg1, params, inputs_b)
        if cfg.kind == wl.KIND_DOUBLE:
            close_to(np.concatenate([got["y_txt"][b], got["y"][b]]), ref["y_rows"], f"sample {b} y rows")
        else:
            close_to(got["y"][b], ref["y"], f"sample {b} y")
        if cfg.sp_degree > 1:
            for k in ("send_q", "send_k", "send_v", "send_attn"):
                close_to(bits_to_f64(got[k][b].view(np.uint16)), ref[k], f"sample {b} {k}")
        alone = single_sample_outputs(cfg1, params, inputs_b, r)
        for k, v in alone.items():
            a, g = np.ascontiguousarray(v), np.ascontiguousarray(got[k][b])
            assert np.array_equal(a.view(np.uint8), g.view(np.uint8)), f"sample {b}: batched {k} differs from the sample run alone"


@pytest.mark.parametrize("rank", [0, 1])
def test_single_stream_batch(rank):
    """Ragged P=2 share (370 local tokens, 740 joint), three samples, rotary tables shared by the batch."""
    cfg = wl.BlockConfig("mini_b3", wl.KIND_SINGLE, n_blocks=1, d=512, n_heads=4, head_dim=128, f=1024, n_total=740,
                         sp_degree=2, sp_rank=rank, qk_rmsnorm=True, n_chunks=5, rope=True, batch=3)
    batch_vs_oracle_and_single(cfg, r=0.0)
    batch_vs_oracle_and_single(cfg, r=0.5)


def test_single_stream_batch_all_heads_local():
    """P=1: attention writes the projection operand directly, one sample after the other."""
    batch_vs_oracle_and_single(wl.CONFIGS["toy"].with_(n_blocks=1, batch=2))


@pytest.mark.parametrize("sp", [1, 2])
def test_dit_cross_batch(sp):
    """Self-attention, cross-attention to a per-sample text context, MLP; two samples."""
    cfg = wl.BlockConfig("mini_dit_b2", wl.KIND_DIT, n_blocks=1, d=512, n_heads=4, head_dim=128, f=1024, n_total=600,
                         sp_degree=sp, sp_rank=sp - 1, l_ctx=77, qk_rmsnorm=True, n_chunks=4, batch=2)
    batch_vs_oracle_and_single(cfg)


@pytest.mark.parametrize("sp", [1, 2])
def test_double_stream_batch(sp):
    """Per-stream weights, joint attention; with a batch the two streams' rows live in separate
    regions, so the attention rows always go through the gather."""
    cfg = wl.BlockConfig("mini_dbl_b2", wl.KIND_DOUBLE, n_blocks=1, d=512, n_heads=8, head_dim=64, f=1024, n_total=576,
                         sp_degree=sp, sp_rank=0, n_txt=64, qk_rmsnorm=True, n_chunks=4, batch=2)
    batch_vs_oracle_and_single(cfg)


def test_mixed_stack_batch_shares_one_strided_residual_buffer():
    """Double-stream then single-stream blocks on a batch: the residual stream is one
    [B, n_local, d] buffer of text-then-image rows per block boundary; the double-stream blocks
    take its text rows and image rows as two views with a sample stride of n_local * d."""
    cfg = wl.CONFIGS["toy_mm"].with_(batch=2)
    L, tl, nl, d, Bn = cfg.n_blocks, cfg.n_txt_local, cfg.n_local, cfg.d, cfg.batch
    run = BlockRunner(cfg)
    try:
        run.ctx.set_resident_fraction(0.0)
        tens = []
        for b in range(L):
            cb = cfg.block_cfg(b)
            run.register_params(b, wl.gen_block_params(cb, b))
            tens.append(run.make_io(wl.gen_block_inputs(cb, b)))
        in0 = wl.gen_block_inputs(cfg.block_cfg(0), 0)
        x0 = np.concatenate([in0["x_txt"], in0["x"]], axis=1)                 # [B, nl, d]
        bufs = [torch.from_numpy(x0).to(run.device)] + [torch.empty((Bn, nl, d), device=run.device) for _ in range(L)]
        for b in range(L):
            t = tens[b]
            if cfg.kind_of(b) == wl.KIND_DOUBLE:
                t["x_txt"], t["x"] = bufs[b][0, :tl], bufs[b][0, tl:]          # pointers of sample 0's rows
                t["y_txt"], t["y"] = bufs[b + 1][0, :tl], bufs[b + 1][0, tl:]
                t["x_sample_stride"] = t["x_txt_sample_stride"] = nl * d
            else:
                t["x"], t["y"] = bufs[b], bufs[b + 1]
        ios = [run.io_struct(t) for t in tens]
        say(f"[toy_mm batch {Bn}] chained stack")
        run.begin(0)
        for b in range(L):
            if b + 1 < L:
                run.begin(b + 1)
            run.fwd(b, ios[b])
        run.ctx.cf_sync()
        got = bufs[L].cpu().numpy()
    finally:
        run.close()
    for s in range(Bn):
        x = x0[s].astype(np.float64)
        for b in range(L):
            cb = cfg.block_cfg(b).with_(batch=1)
            params, inputs = wl.gen_block_params(cb, b), wl.gen_block_inputs(cfg.block_cfg(b), b, sample=s)
            if cb.kind == wl.KIND_DOUBLE:
                x = ob.block_forward(cb, params, dict(inputs, x_txt=x[:tl], x=x[tl:]))["y_rows"]
            else:
                x = ob.block_forward(cb, params, dict(inputs, x=x))["y"]
        r, m = rel_l2(got[s], x), max_abs(got[s], x)
        say(f"   sample {s}: rel_l2={r:.3e} max_abs={m:.3e}")
        assert r <= REL_L2_TOL and m <= 3 * MAX_ABS_TOL            # error adds up over 3 blocks


def test_batch_argument_errors():
    cfg = wl.CONFIGS["toy"]
    with pytest.raises(B.ChunkflowError):
        B.Context(B.desc_from_config(cfg.with_(batch=-1), 1 << 20))
    run = BlockRunner(cfg.with_(batch=2), n_blocks=1)
    try:
        run.register_params(0, wl.gen_block_params(cfg, 0))
        t = run.make_io(wl.gen_block_inputs(cfg.with_(batch=2), 0))
        t["x_sample_stride"] = cfg.n_local * cfg.d - 4             # samples would overlap
        run.begin(0)
        with pytest.raises(B.ChunkflowError) as e:
            run.fwd(0, run.io_struct(t))
        assert e.value.code == B.CF_ERR_ARG
        t["x_sample_stride"] = 0
        run.fwd(0, run.io_struct(t))
        run.ctx.cf_sync()
    finally:
        run.close()
