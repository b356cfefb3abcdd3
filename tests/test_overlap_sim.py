"""The chunk-level walk of the copy and compute streams (Sec. 3.1-3.3).  The oracle's version is
pinned by what the first-order model fixes -- one chunk per block gives max(T_comp, T_pref) per
block (Eq. 1-3), everything resident gives the compute time, no compute gives the transfer time,
weight memory is r*L*W + 2*(1-r)*W at chunk-aligned r (Sec. 3.3) -- and by a case worked by hand.
The library's cf_simulate / cf_tune are then compared with the oracle."""
import numpy as np
import pytest

import workload as wl
from oracle import chunks as oc
from oracle import overlap_model as om
from paper_2605_11335_amd import binding as B
from paper_2605_11335_amd.runner import make_context


def stack(cfg, chunk_bytes, t_comp):
    """Oracle-side description of a stack: per block its blob size, compute time, chunk shares."""
    out = []
    for b in range(cfg.n_blocks):
        cb = cfg.block_cfg(b)
        lay, blob = oc.blob_layout(cb)
        out.append(dict(blob_bytes=blob, t_comp_ms=t_comp[cb.kind], shares=om.segment_shares(cb, lay, blob, chunk_bytes)))
    return out


def test_layout_of_the_library_is_the_oracles():
    for name in ("toy", "flux", "wan", "hunyuan", "toy_mm"):
        cfg = wl.CONFIGS[name].with_(n_blocks=3, n_double=min(1, wl.CONFIGS[name].n_double))
        ctx = make_context(cfg, 1 << 20)
        try:
            for b in range(cfg.n_blocks):
                lay, blob = oc.blob_layout(cfg.block_cfg(b))
                got = [(t["name"], t["offset"], t["rows"], t["cols"]) for t in ctx.cf_blob_layout(b)]
                assert got == lay and ctx.cf_blob_bytes(b) == blob
        finally:
            ctx.close()


def test_one_chunk_per_block_is_the_first_order_closure():
    """Eq. 1-3: hidden iff T_comp >= T_pref; the step is the sum over blocks of the larger."""
    plat = om.Platform(p_peak=1e12, bw_h2d=50e9, eta_comp=1.0, eta_pref=1.0)
    blob = 100_000_000                       # T_pref = 2 ms at 50 GB/s
    for t_comp in (0.5, 2.0, 3.7):
        blocks = [dict(blob_bytes=blob, t_comp_ms=t_comp, shares=[1.0]) for _ in range(5)]
        step, exposed, mem = om.simulate_step(blocks, blob, 0.0, 50.0)
        assert step == pytest.approx(5 * max(t_comp, 2.0), rel=1e-12)
        assert step == pytest.approx(om.step_time(t_comp * 1e-3, blob, 5, plat) * 1e3, rel=1e-12)
        assert exposed == pytest.approx(5 * max(0.0, 2.0 - t_comp), abs=1e-9)
        assert mem == 2 * blob


def test_limits_and_monotonicity():
    cfg = wl.CONFIGS["flux"].with_(n_blocks=4)
    chunk = 32 << 20
    blocks = stack(cfg, chunk, {0: 0.7})
    blob = blocks[0]["blob_bytes"]
    step1, exp1, mem1 = om.simulate_step(blocks, chunk, 1.0, 55.0)
    assert step1 == pytest.approx(4 * 0.7) and abs(exp1) < 1e-12 and mem1 == 4 * blob
    fast = [dict(b, t_comp_ms=1e-9) for b in blocks]
    step0, _, _ = om.simulate_step(fast, chunk, 0.0, 55.0, chunk_overhead_us=10.0)
    n_chunks = -(-blob // chunk)
    assert step0 == pytest.approx(4 * (blob / 55e9 * 1e3 + n_chunks * 0.010), rel=1e-6)
    prev = None
    for r in np.linspace(0, 1, 10):
        step, _, mem = om.simulate_step(blocks, chunk, float(r), 55.0)
        assert prev is None or step <= prev + 1e-12
        prev = step
    # Sec. 3.3 at a chunk-aligned fraction: resident share of every block + two slots for the rest
    n_res = oc.n_resident(n_chunks, 0.5)
    res = n_res * chunk
    assert om.simulate_step(blocks, chunk, 0.5, 55.0)[2] == 4 * res + 2 * (blob - res)
    assert om.weight_memory(blob, 4, res / blob) == pytest.approx(4 * res + 2 * (blob - res))


def test_case_worked_by_hand():
    """Two blocks, two chunks each (1 ms per chunk on the link), compute 1.5 ms per block split
    1 : 2 over the chunks.  Steady state, link-bound: block i's chunks land at 2i+1 and 2i+2 ms
    (the link never idles: the slot's last tenant is long done), its first segment (0.5 ms) starts
    at 2i+1, its second (1 ms) when chunk 2 lands at 2i+2 and ends at 2i+3.  A block ends 1 ms
    after its last chunk lands, the step is 4 ms, 1 ms of it exposed."""
    bytes_per_ms = 1_000_000
    blocks = [dict(blob_bytes=2 * bytes_per_ms, t_comp_ms=1.5, shares=[1 / 3, 2 / 3]) for _ in range(2)]
    step, exposed, mem = om.simulate_step(blocks, bytes_per_ms, 0.0, 1.0)      # 1 GB/s = 1e6 B/ms
    assert step == pytest.approx(4.0) and exposed == pytest.approx(1.0) and mem == 4 * bytes_per_ms
    # first chunk resident: only chunk 2 (1 ms) streams; compute 1.5 ms per block hides it
    step, exposed, mem = om.simulate_step(blocks, bytes_per_ms, 0.5, 1.0)
    assert step == pytest.approx(3.0) and abs(exposed) < 1e-12 and mem == 2 * bytes_per_ms + 2 * bytes_per_ms


@pytest.mark.parametrize("name,blocks,t_comp", [("toy", 2, {0: 0.07}), ("flux", 8, {0: 0.73}), ("wan", 6, {1: 9.1}),
                                                ("hunyuan", 4, {2: 93.0}), ("flux_mm", 6, {0: 0.73, 2: 1.3}),
                                                ("toy_mm", 3, {0: 0.05, 2: 0.12})])
def test_library_simulation_matches_the_oracle(name, blocks, t_comp):
    base = wl.CONFIGS[name]
    cfg = base.with_(n_blocks=blocks, n_double=(max(1, round(blocks * base.n_double / base.n_blocks)) if base.n_double else 0))
    for chunk in (4 << 20, 16 << 20, 64 << 20):
        ctx = make_context(cfg, chunk)
        try:
            st = stack(cfg, chunk, t_comp)
            for r in (0.0, 0.3, 0.5, 0.8, 1.0):
                for ovh in (0.0, 12.0):
                    want = om.simulate_step(st, chunk, r, 55.5, ovh)
                    got = ctx.cf_simulate(r, t_comp, 55.5, ovh)
                    assert got["step_ms"] == pytest.approx(want[0], rel=1e-9)
                    assert got["exposed_ms"] == pytest.approx(want[1], rel=1e-6, abs=1e-9)
                    assert got["weight_memory_bytes"] == want[2]
        finally:
            ctx.close()


def test_tuner_picks_the_best_feasible_point():
    cfg = wl.CONFIGS["flux"]
    cands = [4 << 20, 16 << 20, 64 << 20, 256 << 20]
    ctx = make_context(cfg, 16 << 20)
    try:
        t_comp, link, ovh, steps = {0: 0.73}, 55.5, 12.0, 8
        grid = []
        for c in cands:
            st = stack(cfg, c, t_comp)
            for i in range(steps + 1):
                step, _, mem = om.simulate_step(st, c, i / steps, link, ovh)
                grid.append((c, i / steps, step, mem))
        budget = int(1.2e9)
        ok = [g for g in grid if g[3] <= budget]
        best = min(ok, key=lambda g: (g[2], g[3]))
        got = ctx.cf_tune(t_comp, link, cands, steps, memory_budget_bytes=budget, chunk_overhead_us=ovh)
        assert got["feasible"] and got["weight_memory_bytes"] <= budget
        assert got["step_ms"] == pytest.approx(best[2], rel=1e-9) and got["weight_memory_bytes"] == best[3]
        target = 12.0
        ok = [g for g in grid if g[2] <= target]
        best = min(ok, key=lambda g: (g[3], g[2]))
        got = ctx.cf_tune(t_comp, link, cands, steps, step_target_ms=target, chunk_overhead_us=ovh)
        assert got["feasible"] and got["step_ms"] <= target and got["weight_memory_bytes"] == best[3]
        # nothing fits in 100 MB: the closest point is reported as infeasible
        got = ctx.cf_tune(t_comp, link, cands, steps, memory_budget_bytes=100_000_000, chunk_overhead_us=ovh)
        assert not got["feasible"]
        with pytest.raises(B.ChunkflowError):
            ctx.cf_tune(t_comp, link, cands, steps)                     # neither constraint
        with pytest.raises(B.ChunkflowError):
            ctx.cf_tune(t_comp, link, cands, steps, memory_budget_bytes=budget, step_target_ms=target)
    finally:
        ctx.close()


def test_simulation_argument_errors():
    cfg = wl.CONFIGS["toy"]
    ctx = make_context(cfg, 1 << 20)
    try:
        with pytest.raises(B.ChunkflowError):
            ctx.cf_simulate(1.5, 0.1, 50.0)                      # fraction outside [0, 1]
        with pytest.raises(B.ChunkflowError):
            ctx.cf_simulate(0.5, 0.1, 0.0)                       # no link rate
        with pytest.raises(B.ChunkflowError):
            ctx.cf_simulate(0.5, 0.0, 50.0)                      # no compute time for the model's kind
        with pytest.raises(B.ChunkflowError):
            ctx.cf_simulate(0.5, 0.1, 50.0, chunk_overhead_us=-1.0)
        with pytest.raises(B.ChunkflowError):
            ctx.cf_tune(0.1, 50.0, [1000], 4, memory_budget_bytes=1 << 30)      # chunk size not a multiple of 256
        # a model of one kind ignores the compute times of the others
        only = ctx.cf_simulate(0.0, {0: 0.1}, 50.0)
        more = ctx.cf_simulate(0.0, {0: 0.1, 1: 9.0, 2: 9.0}, 50.0)
        assert only == more
    finally:
        ctx.close()


def test_segment_shares_against_a_layout_worked_by_hand():
    """The booking rule of the chunk-level walk, applied on paper to two matrices and three chunks.

    65536 tokens (256 token tiles, so a row group is 256 output features), one head of 64.
    "w1"  512 x 64  at byte 0      (65536 bytes): rows 0-255 end at byte 32767 (chunk 0), rows 256-511 at 65535 (chunk 1)
    "w2"  256 x 128 at byte 65536  (65536 bytes): one group, ends at byte 131071 (chunk 2)
    chunks of 49152 bytes: [0, 49152), [49152, 98304), [98304, 131072)
    FLOPs (App. B, 2 x tokens x out x in per linear term, 4 x H x N^2 x hd for attention, booked where QKV completes):
      chunk 0: 2 * 65536 * 256 * 64                      = 2,147,483,648
      chunk 1: 2 * 65536 * 256 * 64 + 4 * 65536^2 * 64   = 2,147,483,648 + 1,099,511,627,776
      chunk 2: 2 * 65536 * 256 * 128                     = 4,294,967,296"""
    from types import SimpleNamespace
    cfg = SimpleNamespace(kind=0, n_total=65536, sp_degree=1, n_txt=0, n_heads=1, head_dim=64, l_ctx=0, batch=1)
    lay = [("w1", 0, 512, 64), ("w2", 65536, 256, 128)]
    got = om.segment_shares(cfg, lay, 131072, 49152)
    f = [2_147_483_648, 2_147_483_648 + 1_099_511_627_776, 4_294_967_296]
    assert got == pytest.approx([v / sum(f) for v in f], rel=1e-12)
    # the same matrices under names that carry no attention term: pure linear terms, 1 : 1 : 2
    lay = [("w_o", 0, 512, 64), ("w_up", 65536, 256, 128)]
    assert om.segment_shares(cfg, lay, 131072, 49152) == pytest.approx([0.25, 0.25, 0.5], rel=1e-12)
    # few token tiles: 512 tokens are 2 tiles, a group is 256 * 128 features, so each matrix is one group booked
    # on the chunk of its last byte: w_o (2 * 512 * 512 * 64) on chunk 1, w_up (2 * 512 * 256 * 128) on chunk 2
    small = SimpleNamespace(kind=0, n_total=512, sp_degree=1, n_txt=0, n_heads=1, head_dim=64, l_ctx=0, batch=1)
    assert om.segment_shares(small, lay, 131072, 49152) == pytest.approx([0.0, 0.5, 0.5], rel=1e-12)
    # the modulation matrix multiplies one vector and is booked 8 rows at a time: 24 x 1024 at byte 0 with
    # 16384-byte chunks puts 8 rows (2 * 8 * 1024 FLOPs) on each of three chunks
    lay = [("w_mod", 0, 24, 1024)]
    assert om.segment_shares(small, lay, 49152, 16384) == pytest.approx([1 / 3, 1 / 3, 1 / 3], rel=1e-12)
    # a sharded double-stream block: text-stream matrices see the text rows, image-stream ones the image rows
    dbl = SimpleNamespace(kind=2, n_total=1024, sp_degree=2, n_txt=256, n_heads=2, head_dim=64, l_ctx=0, batch=1)
    lay = [("txt_w_o", 0, 256, 64), ("img_w_o", 32768, 256, 64)]
    # 128 text rows, 384 image rows: 2 * 128 * 256 * 64 on chunk 0, 2 * 384 * 256 * 64 on chunk 1
    assert om.segment_shares(dbl, lay, 65536, 32768) == pytest.approx([0.25, 0.75], rel=1e-12)
