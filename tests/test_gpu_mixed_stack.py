"""A stack that mixes block kinds the way an MMDiT denoiser does (App. B): double-stream blocks,
then single-stream blocks over the concatenated text+image rows.  Every block is checked against
the oracle on its own inputs, the chained stack against the chained oracle (the two kinds share
one residual buffer), and the offloaded arm against the resident one bit for bit."""
import sys

import numpy as np
import pytest
import torch

import workload as wl
from oracle import block as ob
from oracle import chunks as oc
from paper_2605_11335_amd.runner import BlockRunner
from tests.util import max_abs, rel_l2

pytestmark = pytest.mark.gpu
REL_L2_TOL, MAX_ABS_TOL = 1e-2, 5e-2


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def y_rows(cfg_b, t):
    """A block's output rows in joint local order: text rows, then image rows."""
    if cfg_b.kind == wl.KIND_DOUBLE:
        return np.concatenate([t["y_txt"].cpu().numpy(), t["y"].cpu().numpy()])
    return t["y"].cpu().numpy()


@pytest.mark.parametrize("rank", [0, 1])
def test_each_block_of_a_mixed_stack_matches_the_oracle(rank):
    cfg = wl.CONFIGS["toy_mm"].with_(sp_rank=rank)
    run = BlockRunner(cfg)
    try:
        assert [run.ctx.cf_block_kind_of(b) for b in range(cfg.n_blocks)] == cfg.kinds
        run.ctx.set_resident_fraction(0.0)
        for b in range(cfg.n_blocks):
            cb = cfg.block_cfg(b)
            params, inputs = wl.gen_block_params(cb, b), wl.gen_block_inputs(cb, b)
            run.register_params(b, params)
            t = run.make_io(inputs)
            say(f"[toy_mm rank {rank}] block {b} kind {cb.kind}")
            run.run_block(b, t)
            ref = ob.block_forward(cb, params, inputs)
            want = ref["y_rows"] if cb.kind == wl.KIND_DOUBLE else ref["y"]
            got = y_rows(cb, t)
            say(f"   rel_l2={rel_l2(got, want):.3e} max_abs={max_abs(got, want):.3e}")
            assert rel_l2(got, want) <= REL_L2_TOL and max_abs(got, want) <= MAX_ABS_TOL
            # the bytes that landed are the bytes that were registered, chunk by chunk
            host = run.blobs[b].numpy()
            assert run.ctx.cf_n_chunks(b) == len(oc.chunk_bounds(host.size, run.chunk_bytes))
            assert list(run.ctx.cf_checksum_block(b, run.compute)) == list(oc.chunk_checksums(host, run.chunk_bytes))
    finally:
        run.close()


def chained(cfg, r, tens_out=None):
    """Run the whole stack with one shared residual buffer [text rows; image rows] per block
    boundary; returns the final rows."""
    run = BlockRunner(cfg)
    try:
        run.ctx.set_resident_fraction(r)
        L, tl = cfg.n_blocks, cfg.n_txt_local
        tens = []
        for b in range(L):
            cb = cfg.block_cfg(b)
            run.register_params(b, wl.gen_block_params(cb, b))
            tens.append(run.make_io(wl.gen_block_inputs(cb, b)))
        # residual buffers between blocks: buf[b] is read by block b, buf[b+1] written by it
        x0 = np.concatenate([wl.gen_block_inputs(cfg.block_cfg(0), 0)[k] for k in ("x_txt", "x")])
        bufs = [torch.from_numpy(x0).to(run.device)] + [torch.empty((cfg.n_local, cfg.d), device=run.device) for _ in range(L)]
        for b in range(L):
            if cfg.kind_of(b) == wl.KIND_DOUBLE:
                tens[b]["x_txt"], tens[b]["x"] = bufs[b][:tl], bufs[b][tl:]
                tens[b]["y_txt"], tens[b]["y"] = bufs[b + 1][:tl], bufs[b + 1][tl:]
            else:
                tens[b]["x"], tens[b]["y"] = bufs[b], bufs[b + 1]
        ios = [run.io_struct(t) for t in tens]
        run.begin(0)
        run.step(ios)
        run.fwd(0, ios[0])                         # consume the prefetch the last block issued
        run.ctx.cf_sync()
        # block 0 ran twice on the same input: its output is unchanged, the chain's end is bufs[L]
        return bufs[L].cpu().numpy(), x0
    finally:
        run.close()


def test_chained_mixed_stack_matches_the_chained_oracle_and_offload_is_bit_identical():
    cfg = wl.CONFIGS["toy_mm"]
    got, x0 = chained(cfg, 1.0)
    tl = cfg.n_txt_local
    x = x0.astype(np.float64)
    for b in range(cfg.n_blocks):
        cb = cfg.block_cfg(b)
        params, inputs = wl.gen_block_params(cb, b), wl.gen_block_inputs(cb, b)
        if cb.kind == wl.KIND_DOUBLE:
            inputs = dict(inputs, x_txt=x[:tl], x=x[tl:])
            x = ob.block_forward(cb, params, inputs)["y_rows"]
        else:
            x = ob.block_forward(cb, params, dict(inputs, x=x))["y"]
    say(f"[toy_mm chain] rel_l2={rel_l2(got, x):.3e} max_abs={max_abs(got, x):.3e}")
    assert rel_l2(got, x) <= REL_L2_TOL and max_abs(got, x) <= 3 * MAX_ABS_TOL     # error adds up over 3 blocks
    for r in (0.0, 0.5):
        off, _ = chained(cfg, r)
        assert np.array_equal(off.view(np.uint32), got.view(np.uint32)), f"offloaded (r={r}) differs from resident"


def test_flux_like_double_stream_block_at_full_size():
    """The double-stream block of the Flux-like MMDiT share at its real shape (256 text + 2048 image rows of this
    rank, joint attention of 12 heads over 4608 positions, 679 MB of weights streamed in chunks), against the
    oracle's full computation: both streams' outputs and everything this rank would send."""
    from paper_2605_11335_amd.runner import bits_of
    from tests.util import bits_to_f64
    cfg = wl.CONFIGS["flux_mm"].with_(n_blocks=1, n_double=1)
    cb = cfg.block_cfg(0)
    assert cb.kind == wl.KIND_DOUBLE
    params, inputs = wl.gen_block_params(cb, 0), wl.gen_block_inputs(cb, 0)
    run = BlockRunner(cfg)
    try:
        run.ctx.set_resident_fraction(0.0)
        run.register_params(0, params)
        t = run.make_io(inputs)
        say("[flux_mm double-stream, full size] gpu forward")
        run.run_block(0, t)
        say("[flux_mm double-stream, full size] oracle")
        ref = ob.block_forward(cb, params, inputs)
        got = y_rows(cb, t)
        x = np.concatenate([inputs["x_txt"], inputs["x"]])
        r_, m_, rb = rel_l2(got, ref["y_rows"]), max_abs(got, ref["y_rows"]), rel_l2(got - x, ref["y_rows"] - x)
        say(f"   y rel_l2={r_:.3e} max_abs={m_:.3e} branch rel_l2={rb:.3e}")
        assert r_ <= REL_L2_TOL and m_ <= MAX_ABS_TOL and rb <= 2e-2
        for k in ("send_q", "send_k", "send_v", "send_attn"):
            g = bits_to_f64(bits_of(t[k]))
            assert g.shape == ref[k].shape, k
            assert rel_l2(g, ref[k]) <= REL_L2_TOL and max_abs(g, ref[k]) <= MAX_ABS_TOL, k
    finally:
        run.close()
