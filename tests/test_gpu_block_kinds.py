"""Parity of the DiT (cross-attention) and double-stream block forwards, at small sizes against
the full oracle and at the benchmark configurations' full sizes against an exact row sample:
keys and values are built by the oracle for all N tokens, then sampled query rows attend over
all keys exactly and go through the rest of the block exactly."""
import sys

import numpy as np
import pytest

import workload as wl
from oracle import block as ob
from paper_2605_11335_amd.runner import BlockRunner, bits_of
from tests.util import bits_to_f64, max_abs, rel_l2

pytestmark = pytest.mark.gpu
REL_L2_TOL, MAX_ABS_TOL = 1e-2, 5e-2


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run_case(cfg, r=0.0, n_rows=None, seed=0):
    say(f"[{cfg.name}] generating inputs")
    params, inputs = wl.gen_block_params(cfg, 0), wl.gen_block_inputs(cfg, 0)
    run = BlockRunner(cfg, n_blocks=1)
    try:
        run.ctx.set_resident_fraction(r)
        run.register_params(0, params)
        t = run.make_io(inputs)
        say(f"[{cfg.name}] gpu forward")
        run.run_block(0, t)
        rows = send_rows = None
        if n_rows:
            rng = np.random.default_rng(seed)
            rows = np.sort(rng.choice(cfg.n_local, n_rows, replace=False))
            send_rows = np.sort(rng.choice(cfg.n_total - cfg.n_local, 64, replace=False))
        say(f"[{cfg.name}] oracle")
        ref = ob.block_forward(cfg, params, inputs, rows=rows, send_rows=send_rows)
        if cfg.kind == wl.KIND_DOUBLE:
            got = np.concatenate([t["y_txt"].cpu().numpy(), t["y"].cpu().numpy()])
            x = np.concatenate([inputs["x_txt"], inputs["x"]])
            want = ref["y_rows"]
        else:
            got, x, want = t["y"].cpu().numpy(), inputs["x"], ref["y"]
        if rows is not None:
            got, x = got[rows], x[rows]
        r_, m_, rb = rel_l2(got, want), max_abs(got, want), rel_l2(got - x, want - x)
        say(f"[{cfg.name}] y rel_l2={r_:.3e} max_abs={m_:.3e} branch rel_l2={rb:.3e}")
        assert r_ <= REL_L2_TOL and m_ <= MAX_ABS_TOL and rb <= 2e-2
        if cfg.sp_degree > 1:
            sa = bits_to_f64(bits_of(t["send_attn"]))
            if send_rows is not None:
                sa = sa[:, send_rows]
            assert rel_l2(sa, ref["send_attn"]) <= REL_L2_TOL and max_abs(sa, ref["send_attn"]) <= MAX_ABS_TOL
            for k in ("send_q", "send_k", "send_v"):
                g = bits_to_f64(bits_of(t[k]))
                if k == "send_q" and rows is not None:
                    g = g[:, rows]                         # the oracle computes queries of the sampled rows only
                assert g.shape == ref[k].shape, (k, g.shape, ref[k].shape)
                assert rel_l2(g, ref[k]) <= REL_L2_TOL and max_abs(g, ref[k]) <= MAX_ABS_TOL, k
    finally:
        run.close()


@pytest.mark.parametrize("P,rank", [(1, 0), (2, 0), (2, 1)])
def test_dit_block_small(P, rank):
    cfg = wl.BlockConfig("mini_dit", wl.KIND_DIT, n_blocks=1, d=512, n_heads=4, head_dim=128, f=1024,
                         n_total=588, sp_degree=P, sp_rank=rank, l_ctx=77, qk_rmsnorm=True, n_chunks=6)
    run_case(cfg)
    run_case(cfg, r=0.5)


@pytest.mark.parametrize("P,rank", [(1, 0), (2, 0), (2, 1)])
def test_double_stream_block_small(P, rank):
    cfg = wl.BlockConfig("mini_double", wl.KIND_DOUBLE, n_blocks=1, d=512, n_heads=8, head_dim=64, f=1024,
                         n_total=660, sp_degree=P, sp_rank=rank, n_txt=60, qk_rmsnorm=True, n_chunks=9)
    run_case(cfg)
    run_case(cfg, r=0.3)


def _block_outputs(cfg, r):
    params, inputs = wl.gen_block_params(cfg, 0), wl.gen_block_inputs(cfg, 0)
    run = BlockRunner(cfg, n_blocks=1)
    try:
        run.ctx.set_resident_fraction(r)
        run.register_params(0, params)
        t = run.make_io(inputs)
        run.run_block(0, t)
        return {k: v.cpu().numpy().copy() for k, v in t.items() if k in ("y", "y_txt", "send_q", "send_k", "send_v", "send_attn")}
    finally:
        run.close()


@pytest.mark.parametrize("kind", [wl.KIND_DIT, wl.KIND_DOUBLE])
def test_paired_launches_change_no_bit(kind):
    """With every chunk resident the two streams' layers of a double-stream block, and the query /
    context projections of the cross-attention, go out as one launch per pair; while the weights stream
    every layer has its own panel launches.  Same tiles, same k order: the outputs are identical, and
    the resident (paired) arm matches the oracle like the streamed one."""
    if kind == wl.KIND_DIT:
        cfg = wl.BlockConfig("mini_dit", wl.KIND_DIT, n_blocks=1, d=512, n_heads=4, head_dim=128, f=1024,
                             n_total=588, sp_degree=2, sp_rank=1, l_ctx=77, qk_rmsnorm=True, n_chunks=6)
    else:
        cfg = wl.BlockConfig("mini_double", wl.KIND_DOUBLE, n_blocks=1, d=512, n_heads=8, head_dim=64, f=1024,
                             n_total=660, sp_degree=2, sp_rank=0, n_txt=60, qk_rmsnorm=True, n_chunks=9)
    run_case(cfg, r=1.0)
    paired, streamed = _block_outputs(cfg, 1.0), _block_outputs(cfg, 0.0)
    for k in paired:
        assert np.array_equal(paired[k].view(np.uint8), streamed[k].view(np.uint8)), k


def test_wan_share_full_size_row_sample():
    """C3: 27280 video tokens, cross-attention to 512 text tokens, P=2 share."""
    run_case(wl.CONFIGS["wan"].with_(n_blocks=1), n_rows=192)


def test_hunyuan_share_full_size_row_sample():
    """C4: joint attention over 118800 video + 256 text tokens, P=2 share (59400 + 128 local rows)."""
    run_case(wl.CONFIGS["hunyuan"].with_(n_blocks=1), n_rows=160)
