"""CPU-side checks of the C ABI: the library loads, exports what the header declares, and the
planning calls (which touch no GPU) behave: layout, chunking, argument errors."""
import ctypes as C
import os
import re

import numpy as np

import itertools

import pytest

import workload as wl
from oracle import chunks as och
from oracle import overlap_model as om
from paper_2605_11335_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions(name=None):
    """Functions declared by include/<name> (every header of include/ when no name is given)."""
    inc = os.path.join(ROOT, "include")
    names = []
    for h in sorted(os.listdir(inc)) if name is None else [name]:
        text = open(os.path.join(inc, h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"^\s*(?:int|const char\*)\s+(\w+)\s*\(", text, flags=re.M)
    return names


def test_library_exports_every_declared_symbol():
    names = header_functions()
    assert len(names) >= 25 and "dit_block_fwd" in names and "set_resident_fraction" in names
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(names) == sorted(B.EXPORTS)
    # the block path's contract and the diagnostics are separate headers
    core, diag = header_functions("chunkflow.h"), header_functions("chunkflow_diag.h")
    assert sorted(core) == sorted(B.CORE_EXPORTS) and sorted(diag) == sorted(B.DIAG_EXPORTS)
    assert not any(n.startswith("cf_op_") or n in ("cf_plan_attention", "cf_plan_linear") for n in core
                   if not n.startswith("cf_op_checksum"))


def ctx_for(cfg, chunk):
    return B.Context(B.desc_from_config(cfg, chunk))


def test_blob_bytes_follow_app_b_formulas():
    flux = wl.CONFIGS["flux"]
    c = ctx_for(flux, 16 << 20)
    extra = c.cf_blob_bytes() - om.bytes_single(flux.d, flux.f)       # biases + norm weights + padding
    assert 0 < extra < 100_000
    hy = wl.CONFIGS["hunyuan"]
    c2 = ctx_for(hy, 16 << 20)
    extra = c2.cf_blob_bytes() - om.bytes_double(hy.d, hy.f)
    assert 0 < extra < 300_000
    wan = wl.CONFIGS["wan"]
    c3 = ctx_for(wan, 16 << 20)
    d, f = wan.d, wan.f
    assert 0 < c3.cf_blob_bytes() - 2 * (6 * d * d + 4 * d * d + 4 * d * d + 2 * d * f) < 300_000


@pytest.mark.parametrize("name", ["toy", "flux", "wan", "hunyuan"])
def test_layout_is_aligned_ordered_and_complete(name):
    cfg = wl.CONFIGS[name]
    c = ctx_for(cfg, 1 << 20)
    lay = c.cf_blob_layout()
    specs = {n: shape for n, shape, _, _ in wl.param_specs(cfg)}
    assert {t["name"] for t in lay} == set(specs)
    end = 0
    for t in lay:
        assert t["offset"] % 256 == 0 and t["offset"] >= end
        shape = specs[t["name"]]
        assert t["rows"] * t["cols"] == int(__import__("numpy").prod(shape))
        if len(shape) == 2:
            assert (t["rows"], t["cols"]) == shape
        end = t["offset"] + 2 * t["rows"] * t["cols"]
    assert end <= c.cf_blob_bytes() < end + 256
    assert c.cf_workspace_bytes() > 0


def test_chunk_count_matches_oracle_arithmetic():
    cfg = wl.CONFIGS["flux"]
    for chunk in (16 << 20, 64 << 20, 256 << 20, 1 << 20):
        c = ctx_for(cfg, chunk)
        assert c.cf_n_chunks() == len(och.chunk_bounds(c.cf_blob_bytes(), chunk))


def test_toy_config_is_four_chunks():
    from paper_2605_11335_amd.runner import chunk_bytes_for
    cfg = wl.CONFIGS["toy"]
    cb = chunk_bytes_for(cfg)
    assert cb % 256 == 0
    assert ctx_for(cfg, cb).cf_n_chunks() == 4
    assert ctx_for(wl.CONFIGS["flux"], chunk_bytes_for(wl.CONFIGS["flux"])).cf_n_chunks() == 8


@pytest.mark.parametrize("field,value", [("chunk_bytes", 0), ("chunk_bytes", 1000), ("head_dim", 96), ("sp_degree", 5),
                                         ("n_total", 4607), ("d", 3000), ("kind", 7), ("n_blocks", 0), ("f", 100),
                                         ("sp_rank", 2)])
def test_create_rejects_bad_descriptions(field, value):
    d = B.desc_from_config(wl.CONFIGS["flux"], 16 << 20)
    setattr(d, field, value)
    with pytest.raises(B.ChunkflowError) as e:
        B.Context(d)
    assert e.value.code == B.CF_ERR_ARG and str(e.value)


def test_block_range_is_checked_without_a_gpu():
    c = ctx_for(wl.CONFIGS["toy"], 1 << 20)
    with pytest.raises(B.ChunkflowError) as e:
        c.chunked_prefetch_begin(5, None)
    assert e.value.code == B.CF_ERR_ARG


@pytest.mark.parametrize("name,chunk_mib", [("flux", 16), ("flux", 35.4), ("wan", 64), ("toy", 0.5), ("hunyuan", 256)])
def test_panel_plans_cover_every_row_once_behind_the_right_chunk(name, chunk_mib):
    """Host logic of the per-chunk consumer waits: for every weight matrix and every resident
    prefix, panels tile the rows exactly, are tile-aligned, and every byte of a panel lies in a
    chunk that is resident or not later than the chunk the panel waits for; for several token
    counts of the layer, since the panel ends depend on how the launch fills the chip."""
    cfg = wl.CONFIGS[name]
    cb = int(chunk_mib * (1 << 20)) // 256 * 256
    c = ctx_for(cfg, cb)
    n_chunks = c.cf_n_chunks()
    bounds = och.chunk_bounds(c.cf_blob_bytes(), cb)
    for t in c.cf_blob_layout():
        if t["rows"] == 1:
            continue
        row_bytes = 2 * t["cols"]
        for n_res, m_rows in itertools.product(sorted({0, 1, n_chunks // 3, n_chunks // 2, n_chunks - 1, n_chunks}),
                                               (0, 1, cfg.n_local, 5 * cfg.n_local)):
            plan = c.cf_plan_panels(t["name"], m_rows, n_res)
            assert plan[0][0] == 0 and plan[-1][1] == t["rows"]
            for (a0, a1, w), nxt in zip(plan, plan[1:] + [None]):
                assert a0 < a1
                if nxt is not None:
                    assert a1 == nxt[0] and a1 % (256 if m_rows else 8) == 0 and w < nxt[2]
                last_byte = t["offset"] + a1 * row_bytes - 1
                need = next(k for k, (s, e) in enumerate(bounds) if s <= last_byte < e)
                assert need < n_res or need <= w, (t["name"], n_res, a0, a1, w, need)
                if w >= 0:
                    assert w >= n_res        # never waits for a resident chunk
            if n_res == n_chunks:
                assert plan == [(0, t["rows"], -1)]     # fully resident: one launch, no wait


def test_panels_fill_their_rounds_of_workgroups():
    """Every launch ends with a partly filled round of workgroups, so a layer is not cut wherever a
    chunk ends.  Flux-like lin1 (84 feature tiles of 256) on 2304 tokens (9 token tiles): 28
    feature tiles make 252 of the 256 workgroups of one round; although a 16 MiB chunk ends every
    10.7 tiles, the first panel leaves at most 7 % of its rounds empty and no panel but the last
    more than a quarter (such a remainder would have stayed with the next panel)."""
    cfg = wl.CONFIGS["flux"]
    c = ctx_for(cfg, 16 << 20)
    plan = c.cf_plan_panels("w1", cfg.n_local, 0)
    assert len(plan) >= 3
    for i, (a0, a1, w) in enumerate(plan[:-1]):
        tiles = (a1 - a0) // 256 * 9
        launched = -(-tiles // 256) * 256
        assert (a1 - a0) % 256 == 0 and launched - tiles <= (0.07 if i == 0 else 0.25) * launched, plan
    # lin2 (12 feature tiles x 9 token tiles): no cut fills a round; one launch behind its last chunk
    plan2 = c.cf_plan_panels("w2", cfg.n_local, 0)
    assert len(plan2) == 1 and plan2[0][:2] == (0, cfg.d)
    # the modulation product is cut at every chunk end
    assert len(c.cf_plan_panels("w_mod", 0, 0)) >= 2 or c.cf_n_chunks() == 1


def test_mixed_block_kinds_are_planned_per_block():
    """App. B composition: double-stream blocks then single-stream ones; each kind has its own
    layout and chunk count, the workspace covers both."""
    cfg = wl.CONFIGS["toy_mm"]
    chunk = 1 << 20
    ctx = B.Context(B.desc_from_config(cfg, chunk))
    try:
        single_bytes, single_ws = ctx.cf_blob_bytes(), ctx.cf_workspace_bytes()
        ctx.cf_set_block_kinds(cfg.kinds)
        assert [ctx.cf_block_kind_of(b) for b in range(cfg.n_blocks)] == [wl.KIND_DOUBLE, wl.KIND_SINGLE, wl.KIND_SINGLE]
        assert ctx.cf_blob_bytes(1) == ctx.cf_blob_bytes(2) == single_bytes
        assert ctx.cf_workspace_bytes() >= single_ws
        for b in range(cfg.n_blocks):
            specs = wl.param_specs(cfg.block_cfg(b))
            lay = ctx.cf_blob_layout(b)
            assert sorted(t["name"] for t in lay) == sorted(s[0] for s in specs)
            want = sum(-(-2 * int(np.prod(s[1])) // 256) * 256 for s in specs)
            assert ctx.cf_blob_bytes(b) == want
            assert ctx.cf_n_chunks(b) == -(-want // chunk)
        with pytest.raises(B.ChunkflowError):
            ctx.cf_set_block_kinds([0, 0])                      # one kind per block
        with pytest.raises(B.ChunkflowError):
            ctx.cf_set_block_kinds([wl.KIND_DIT, 0, 0])         # no cross-attention context in this model
    finally:
        ctx.close()
    no_txt = B.Context(B.desc_from_config(wl.CONFIGS["toy"], chunk))
    try:
        with pytest.raises(B.ChunkflowError):
            no_txt.cf_set_block_kinds([wl.KIND_DOUBLE, 0])      # double-stream needs text rows
    finally:
        no_txt.close()


def test_attention_launch_shapes():
    """The launch planner's choices for the shapes they were measured on (one MI355X): 8 waves per
    workgroup for the Flux-like and the Hunyuan-like self-attention, 7 for the Wan-like one (7- and 8-wave
    grids take six generations either way, and a 7-wave generation of such a long sweep is shorter), 4 for
    the cross-attention to 512 context tokens (short sweeps: one workgroup's fixed part hides behind the
    other's tiles) and for grids that end on a half-empty generation; tiny grids are spread over 4-wave
    workgroups.  Growing the key count alone never moves a choice from 8 towards 4."""
    assert B.cf_plan_attention(12, 4608, 4608, 128) == 8
    assert B.cf_plan_attention(12, 119056, 119056, 128) == 8
    assert B.cf_plan_attention(12, 59528, 59528, 128) == 8
    assert B.cf_plan_attention(12, 27280, 27280, 128) == 7
    assert B.cf_plan_attention(24, 13640, 512, 128) == 4
    assert B.cf_plan_attention(12, 8192, 8192, 128) == 4
    assert B.cf_plan_attention(24, 4096, 4096, 128) == 4
    assert B.cf_plan_attention(8, 512, 512, 64) == 4
    for nq, H in ((4608, 12), (13640, 24), (5120, 8)):
        picks = [B.cf_plan_attention(H, nq, nk, 128) for nk in (128, 512, 2048, 8192, 32768)]
        assert all(p in (4, 7, 8) for p in picks)
        first_tall = next((i for i, p in enumerate(picks) if p != 4), len(picks))
        assert all(p != 4 for p in picks[first_tall:]), picks
    for bad in ((0, 10, 10, 128), (1, 0, 10, 128), (1, 10, 0, 128), (1, 10, 10, 96)):
        with pytest.raises(B.ChunkflowError):
            B.cf_plan_attention(*bad)


def test_linear_tile_shapes():
    """The tile choice for layer shapes on which both tiles were timed (one MI355X, operands read cold): the
    listed choice was the faster one by 5-45 % (the Flux-like and Wan-like shares' layers, the context
    projection of the Wan-like cross-attention, the image stream of the mixed stack's double-stream blocks)."""
    for m, n, want in ((2304, 21504, 256), (2304, 3072, 128), (13640, 3072, 256), (13640, 9216, 256), (2048, 3072, 128),
                       (512, 6144, 128), (4608, 3072, 256), (4608, 9216, 256), (1024, 21504, 256)):
        assert B.cf_plan_linear(m, n) == want, (m, n)
    assert B.cf_plan_linear(64, 64) == 128                       # one tile either way: the small one
    with pytest.raises(B.ChunkflowError):
        B.cf_plan_linear(0, 64)


def test_no_alloc_checksum_rejects_oversize_and_misaligned_requests_before_touching_a_gpu():
    """The argument checks of cf_op_checksum_noalloc come before any HIP call: a request beyond what
    its fixed partial-sum array covers (1 GiB) is an argument error with a message that says so."""
    lib = B.lib()
    fake = C.c_void_p(4096)             # never dereferenced: the call must fail on its arguments
    assert lib.cf_op_checksum_noalloc(fake, (1 << 30) + 8, 0, fake, None) == B.CF_ERR_ARG
    assert b"exceed" in lib.cf_last_error(None)
    assert lib.cf_op_checksum_noalloc(fake, 12, 0, fake, None) == B.CF_ERR_ARG
    assert lib.cf_op_checksum_noalloc(fake, 8, 0, None, None) == B.CF_ERR_ARG
    assert lib.cf_op_checksum_noalloc(C.c_void_p(4097), 8, 0, fake, None) == B.CF_ERR_ARG
