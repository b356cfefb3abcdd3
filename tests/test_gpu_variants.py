"""Block variants beyond the default reading.  Rotary position tables handed to the block: q and k (of every head, including the ones this
rank sends away) are rotated after the per-head norm; cross-attention is not.  All three block
kinds and a mixed stack against the oracle."""
import sys

import numpy as np
import pytest

import workload as wl
from oracle import block as ob
from paper_2605_11335_amd.runner import BlockRunner, bits_of
from tests.util import bits_to_f64, max_abs, rel_l2

pytestmark = pytest.mark.gpu
REL_L2_TOL, MAX_ABS_TOL = 1e-2, 5e-2

CASES = {
    "single": wl.BlockConfig("rope_single", wl.KIND_SINGLE, n_blocks=1, d=512, n_heads=8, head_dim=64, f=1024,
                             n_total=456, sp_degree=2, sp_rank=1, qk_rmsnorm=True, n_chunks=5, rope=True),
    "single_no_norm": wl.BlockConfig("rope_plain", wl.KIND_SINGLE, n_blocks=1, d=512, n_heads=4, head_dim=128, f=1024,
                                     n_total=300, sp_degree=1, qk_rmsnorm=False, n_chunks=3, rope=True),
    "dit": wl.BlockConfig("rope_dit", wl.KIND_DIT, n_blocks=1, d=512, n_heads=4, head_dim=128, f=1024,
                          n_total=588, sp_degree=2, sp_rank=0, l_ctx=77, qk_rmsnorm=True, n_chunks=6, rope=True),
    "double": wl.BlockConfig("rope_double", wl.KIND_DOUBLE, n_blocks=1, d=512, n_heads=8, head_dim=64, f=1024,
                             n_total=660, sp_degree=2, sp_rank=1, n_txt=60, qk_rmsnorm=True, n_chunks=9, rope=True),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_block_with_rotary_tables(name):
    cfg = CASES[name]
    params, inputs = wl.gen_block_params(cfg, 0), wl.gen_block_inputs(cfg, 0)
    assert inputs["rope_cos"].shape == (cfg.n_local, cfg.head_dim // 2)
    run = BlockRunner(cfg)
    try:
        run.ctx.set_resident_fraction(0.4)
        run.register_params(0, params)
        t = run.make_io(inputs)
        print(f"[{cfg.name}] gpu forward", flush=True)
        run.run_block(0, t)
        ref = ob.block_forward(cfg, params, inputs)
        if cfg.kind == wl.KIND_DOUBLE:
            got, want = np.concatenate([t["y_txt"].cpu().numpy(), t["y"].cpu().numpy()]), ref["y_rows"]
        else:
            got, want = t["y"].cpu().numpy(), ref["y"]
        print(f"[{cfg.name}] rel_l2={rel_l2(got, want):.3e} max_abs={max_abs(got, want):.3e}", flush=True)
        assert rel_l2(got, want) <= REL_L2_TOL and max_abs(got, want) <= MAX_ABS_TOL
        # the rotation must matter: the kernel's branch output is far closer to the oracle with the
        # tables than to the oracle without them
        plain = ob.block_forward(cfg, params, {k: v for k, v in inputs.items() if not k.startswith("rope_")})
        plain = plain["y_rows"] if cfg.kind == wl.KIND_DOUBLE else plain["y"]
        x = np.concatenate([inputs["x_txt"], inputs["x"]]) if cfg.kind == wl.KIND_DOUBLE else inputs["x"]
        assert rel_l2(got - x, plain - x) > 5 * rel_l2(got - x, want - x)
        if cfg.sp_degree > 1:
            for k in ("send_q", "send_k", "send_v", "send_attn"):
                g = bits_to_f64(bits_of(t[k]))
                assert rel_l2(g, ref[k]) <= REL_L2_TOL and max_abs(g, ref[k]) <= MAX_ABS_TOL, k
        # one table without the other is an argument error
        bad = dict(t)
        del bad["rope_sin"]
        with pytest.raises(Exception):
            run.run_block(0, bad)
    finally:
        run.close()


@pytest.mark.parametrize("name", ["single", "dit", "double"])
def test_block_with_erf_gelu(name):
    cfg = CASES[name].with_(rope=False, gelu_erf=True, name=CASES[name].name + "_erf")
    params, inputs = wl.gen_block_params(cfg, 0), wl.gen_block_inputs(cfg, 0)
    run = BlockRunner(cfg)
    try:
        run.ctx.set_resident_fraction(0.0)
        run.register_params(0, params)
        t = run.make_io(inputs)
        print(f"[{cfg.name}] gpu forward", flush=True)
        run.run_block(0, t)
        ref = ob.block_forward(cfg, params, inputs)
        tanh = ob.block_forward(cfg.with_(gelu_erf=False), params, inputs)
        if cfg.kind == wl.KIND_DOUBLE:
            got, want, other = np.concatenate([t["y_txt"].cpu().numpy(), t["y"].cpu().numpy()]), ref["y_rows"], tanh["y_rows"]
        else:
            got, want, other = t["y"].cpu().numpy(), ref["y"], tanh["y"]
        print(f"[{cfg.name}] rel_l2={rel_l2(got, want):.3e} max_abs={max_abs(got, want):.3e}", flush=True)
        assert rel_l2(got, want) <= REL_L2_TOL and max_abs(got, want) <= MAX_ABS_TOL
        assert max_abs(want, other) > 0        # the two activations do differ on these inputs
    finally:
        run.close()
