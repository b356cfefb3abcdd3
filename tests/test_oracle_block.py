"""Pins for the oracle's block forwards: special cases with closed-form outcomes, an
independent composition from torch CPU library routines, the P=2 Ulysses shares
reassembling the P=1 block, row sampling, and MAC counts against the App. B formulas."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workload as wl
from oracle import block as ob
from oracle import overlap_model as om


def tiny(kind, P=1, rank=0, qk=True, **kw):
    base = dict(name=f"tiny{kind}", kind=kind, n_blocks=1, d=32, n_heads=4, head_dim=8, f=48,
                n_total=24, sp_degree=P, sp_rank=rank, n_txt=8 if kind == wl.KIND_DOUBLE else 0,
                l_ctx=6 if kind == wl.KIND_DIT else 0, qk_rmsnorm=qk, n_chunks=2)
    base.update(kw)
    return wl.BlockConfig(**base)


def draw(cfg, scale_w=8.0):
    """Seeded params/inputs; weights scaled up so every term matters at these tiny widths."""
    p = {k: ob.widen(v) * (scale_w if ("norm" not in k and not k.startswith("ln_c")) else 1.0)
         for k, v in wl.gen_block_params(cfg, 0).items()}
    i = {k: ob.widen(v) for k, v in wl.gen_block_inputs(cfg, 0).items()}
    return p, i


def T(a):
    return torch.from_numpy(np.ascontiguousarray(a))


def torch_heads_attention(q, k, v, H):
    n, d = q.shape
    sp = lambda z: z.reshape(z.shape[0], H, d // H).transpose(0, 1)
    return F.scaled_dot_product_attention(sp(q), sp(k), sp(v)).transpose(0, 1).reshape(n, d)


def torch_rms(z, w, H):
    if w is None:
        return z
    n, d = z.shape
    zz = z.reshape(n, H, d // H)
    return (zz * torch.rsqrt((zz * zz).mean(-1, keepdim=True) + 1e-6) * w).reshape(n, d)


def torch_single(cfg, p, i):
    d, H = cfg.d, cfg.n_heads
    x, t = T(i["x"]), T(i["temb"])
    m = F.linear(t, T(p["w_mod"]), T(p["b_mod"]))
    shift, scale, gate = m.split(d)
    xn = F.layer_norm(x, (d,), eps=1e-6) * (1 + scale) + shift
    z = F.linear(xn, T(p["w1"]), T(p["b1"]))
    q, k, v, u = z.split([d, d, d, cfg.f], dim=1)
    if cfg.qk_rmsnorm:
        q, k = torch_rms(q, T(p["q_norm"]), H), torch_rms(k, T(p["k_norm"]), H)
    a = torch_heads_attention(q, k, v, H)
    c = torch.cat([a, F.gelu(u, approximate="tanh")], dim=1)
    return (x + gate * F.linear(c, T(p["w2"]), T(p["b2"]))).numpy()


def torch_dit(cfg, p, i):
    d, H = cfg.d, cfg.n_heads
    x, t, ctx = T(i["x"]), T(i["temb"]), T(i["ctx"])
    sh1, sc1, g1, sh2, sc2, g2 = F.linear(t, T(p["w_mod"]), T(p["b_mod"])).split(d)
    h = F.layer_norm(x, (d,), eps=1e-6) * (1 + sc1) + sh1
    q, k, v = F.linear(h, T(p["w_qkv"]), T(p["b_qkv"])).split(d, dim=1)
    q, k = torch_rms(q, T(p["q_norm"]), H), torch_rms(k, T(p["k_norm"]), H)
    x = x + g1 * F.linear(torch_heads_attention(q, k, v, H), T(p["w_o"]), T(p["b_o"]))
    hc = F.layer_norm(x, (d,), T(p["ln_c_w"]), T(p["ln_c_b"]), eps=1e-6)
    qc = torch_rms(F.linear(hc, T(p["w_cq"]), T(p["b_cq"])), T(p["cq_norm"]), H)
    kc, vc = F.linear(ctx, T(p["w_ckv"]), T(p["b_ckv"])).split(d, dim=1)
    kc = torch_rms(kc, T(p["ck_norm"]), H)
    x = x + F.linear(torch_heads_attention(qc, kc, vc, H), T(p["w_co"]), T(p["b_co"]))
    h2 = F.layer_norm(x, (d,), eps=1e-6) * (1 + sc2) + sh2
    up = F.gelu(F.linear(h2, T(p["w_up"]), T(p["b_up"])), approximate="tanh")
    return (x + g2 * F.linear(up, T(p["w_down"]), T(p["b_down"]))).numpy()


def torch_double(cfg, p, i):
    d, H = cfg.d, cfg.n_heads
    t = T(i["temb"])
    xs = {"txt": T(i["x_txt"]), "img": T(i["x"])}
    mods, qkv = {}, {}
    for s in ("txt", "img"):
        mods[s] = F.linear(t, T(p[f"{s}_w_mod"]), T(p[f"{s}_b_mod"])).split(d)
        h = F.layer_norm(xs[s], (d,), eps=1e-6) * (1 + mods[s][1]) + mods[s][0]
        q, k, v = F.linear(h, T(p[f"{s}_w_qkv"]), T(p[f"{s}_b_qkv"])).split(d, dim=1)
        qkv[s] = (torch_rms(q, T(p[f"{s}_q_norm"]), H), torch_rms(k, T(p[f"{s}_k_norm"]), H), v)
    q, k, v = (torch.cat([qkv["txt"][j], qkv["img"][j]]) for j in range(3))
    a = torch_heads_attention(q, k, v, H)
    tl = xs["txt"].shape[0]
    out = {}
    for s, a_s in (("txt", a[:tl]), ("img", a[tl:])):
        sh1, sc1, g1, sh2, sc2, g2 = mods[s]
        x = xs[s] + g1 * F.linear(a_s, T(p[f"{s}_w_o"]), T(p[f"{s}_b_o"]))
        h2 = F.layer_norm(x, (d,), eps=1e-6) * (1 + sc2) + sh2
        up = F.gelu(F.linear(h2, T(p[f"{s}_w_up"]), T(p[f"{s}_b_up"])), approximate="tanh")
        out[s] = (x + g2 * F.linear(up, T(p[f"{s}_w_down"]), T(p[f"{s}_b_down"]))).numpy()
    return out


def test_single_stream_matches_library_composition():
    for qk in (True, False):
        cfg = tiny(wl.KIND_SINGLE, qk=qk)
        p, i = draw(cfg)
        np.testing.assert_allclose(ob.single_stream_block(cfg, p, i)["y"], torch_single(cfg, p, i), rtol=1e-9, atol=1e-11)


def test_dit_matches_library_composition():
    cfg = tiny(wl.KIND_DIT)
    p, i = draw(cfg)
    np.testing.assert_allclose(ob.dit_block(cfg, p, i)["y"], torch_dit(cfg, p, i), rtol=1e-9, atol=1e-11)


def test_double_stream_matches_library_composition():
    cfg = tiny(wl.KIND_DOUBLE)
    p, i = draw(cfg)
    o = ob.double_stream_block(cfg, p, i)
    ref = torch_double(cfg, p, i)
    np.testing.assert_allclose(o["y"], ref["img"], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(o["y_txt"], ref["txt"], rtol=1e-9, atol=1e-11)


def test_identity_adaln_collapses_to_layernorm_plus_residual():
    """shift=0, scale=0, gate=1: the block is x + branch(LayerNorm(x)) with no modulation."""
    cfg = tiny(wl.KIND_SINGLE)
    p, i = draw(cfg)
    d = cfg.d
    p["w_mod"] = np.zeros_like(p["w_mod"])
    p["b_mod"] = np.concatenate([np.zeros(d), np.zeros(d), np.ones(d)])
    x = T(i["x"])
    xn = F.layer_norm(x, (d,), eps=1e-6)
    z = F.linear(xn, T(p["w1"]), T(p["b1"]))
    q, k, v, u = z.split([d, d, d, cfg.f], dim=1)
    q, k = torch_rms(q, T(p["q_norm"]), cfg.n_heads), torch_rms(k, T(p["k_norm"]), cfg.n_heads)
    c = torch.cat([torch_heads_attention(q, k, v, cfg.n_heads), F.gelu(u, approximate="tanh")], dim=1)
    ref = (x + F.linear(c, T(p["w2"]), T(p["b2"]))).numpy()
    np.testing.assert_allclose(ob.single_stream_block(cfg, p, i)["y"], ref, rtol=1e-9, atol=1e-11)


def test_gate_zero_returns_input_and_scale_minus_one_erases_tokens():
    cfg = tiny(wl.KIND_SINGLE)
    p, i = draw(cfg)
    d = cfg.d
    p["w_mod"] = np.zeros_like(p["w_mod"])
    p["b_mod"] = np.concatenate([np.full(d, 0.3), np.full(d, 0.7), np.zeros(d)])
    np.testing.assert_array_equal(ob.single_stream_block(cfg, p, i)["y"], i["x"])
    # scale = -1 wipes LN(x): every token sees xn = shift, so the branch is the same row for all tokens
    p["b_mod"] = np.concatenate([np.linspace(-1, 1, d), np.full(d, -1.0), np.ones(d)])
    br = ob.single_stream_block(cfg, p, i)["y"] - i["x"]
    assert np.abs(br - br[:1]).max() < 1e-9 and np.abs(br).max() > 1e-3


@pytest.mark.parametrize("kind", [wl.KIND_SINGLE, wl.KIND_DIT, wl.KIND_DOUBLE])
def test_two_ulysses_shares_reassemble_the_full_block(kind):
    """Run rank 0 and rank 1 with each other's send buffers as peer buffers (an exchange by
    hand): the stacked outputs must be the P=1 block on the full sequence."""
    full = tiny(kind, P=1)
    pf, inf = draw(full)
    ref = ob.block_forward(full, pf, inf)
    cfgs = [tiny(kind, P=2, rank=r) for r in range(2)]
    N, H, hd, d = full.n_total, full.n_heads, full.head_dim, full.d
    lpos = [ob.local_positions(c) for c in cfgs]
    # local inputs of each rank = its rows of the full input (local order: text rows then image rows)
    def local_inputs(r):
        i = {"temb": inf["temb"]}
        if kind == wl.KIND_DOUBLE:
            tl = full.n_txt // 2
            i["x_txt"] = inf["x_txt"][r * tl:(r + 1) * tl]
            il = (N - full.n_txt) // 2
            i["x"] = inf["x"][r * il:(r + 1) * il]
        else:
            i["x"] = inf["x"][lpos[r]]
        if kind == wl.KIND_DIT:
            i["ctx"] = inf["ctx"]
        return i
    ins = [local_inputs(r) for r in range(2)]
    # pass 1: each rank's q,k,v sends do not depend on its peers
    dummy = lambda c: {"peer_q": np.zeros((H // 2, N // 2, hd)), "peer_k": np.zeros((H // 2, N // 2, hd)),
                       "peer_v": np.zeros((H // 2, N // 2, hd)), "peer_attn": np.zeros((N // 2, H // 2, hd))}
    first = [ob.block_forward(cfgs[r], pf, {**ins[r], **dummy(cfgs[r])}) for r in range(2)]
    # with P=2 the other rank's tokens are exactly the remote positions, in ascending order
    for r in range(2):
        o = 1 - r
        ins[r].update(peer_q=first[o]["send_q"], peer_k=first[o]["send_k"], peer_v=first[o]["send_v"],
                      peer_attn=np.zeros((N // 2, H // 2, hd)))
    second = [ob.block_forward(cfgs[r], pf, ins[r]) for r in range(2)]
    for r in range(2):
        o = 1 - r
        ins[r]["peer_attn"] = second[o]["send_attn"].transpose(1, 0, 2)
    final = [ob.block_forward(cfgs[r], pf, ins[r]) for r in range(2)]
    if kind == wl.KIND_DOUBLE:
        np.testing.assert_allclose(np.concatenate([final[0]["y_txt"], final[1]["y_txt"]]), ref["y_txt"], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(np.concatenate([final[0]["y"], final[1]["y"]]), ref["y"], rtol=1e-9, atol=1e-11)
    else:
        np.testing.assert_allclose(np.concatenate([final[0]["y"], final[1]["y"]]), ref["y"], rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("kind", [wl.KIND_SINGLE, wl.KIND_DIT, wl.KIND_DOUBLE])
def test_row_sampling_equals_full_rows(kind):
    cfg = tiny(kind, P=2, rank=1)
    p, i = draw(cfg)
    full = ob.block_forward(cfg, p, i)
    rows, srows = np.array([0, 3, 5, 11]), np.array([1, 7])
    part = ob.block_forward(cfg, p, i, rows=rows, send_rows=srows)
    if kind == wl.KIND_DOUBLE:
        np.testing.assert_allclose(part["y_rows"], full["y_rows"][rows], rtol=1e-10, atol=1e-12)
    else:
        np.testing.assert_allclose(part["y"], full["y"][rows], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(part["send_attn"], full["send_attn"][:, srows], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(part["send_k"], full["send_k"], rtol=1e-12)


def test_mac_counts_match_app_b():
    P = 2
    # single-stream: every term divides by the SP degree
    cfg = tiny(wl.KIND_SINGLE, P=P)
    p, i = draw(cfg)
    mc = ob.MacCounter()
    ob.block_forward(cfg, p, i, mc=mc)
    assert mc.flops() * P == om.flops_single(1, cfg.n_total, cfg.d, cfg.f, 0)
    assert mc.flops("lin1") * P == 2 * cfg.n_total * cfg.d * (3 * cfg.d + cfg.f)
    assert mc.flops("attn") * P == 4 * cfg.n_total ** 2 * cfg.d
    # DiT: the text-side K/V projection is replicated on every rank, all else divides
    cfg = tiny(wl.KIND_DIT, P=P)
    p, i = draw(cfg)
    mc = ob.MacCounter()
    ob.block_forward(cfg, p, i, mc=mc)
    rep = mc.flops("cross_kv")
    assert rep == 4 * cfg.l_ctx * cfg.d ** 2
    assert (mc.flops() - rep) * P + rep == om.flops_dit(1, cfg.n_total, cfg.d, cfg.f, cfg.l_ctx)
    # double-stream: S image tokens + L text tokens
    cfg = tiny(wl.KIND_DOUBLE, P=P)
    p, i = draw(cfg)
    mc = ob.MacCounter()
    ob.block_forward(cfg, p, i, mc=mc)
    assert mc.flops() * P == om.flops_double(1, cfg.n_total - cfg.n_txt, cfg.d, cfg.f, cfg.n_txt)
