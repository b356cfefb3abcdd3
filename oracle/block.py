"""CPU oracle for one GPU's Ulysses share of a DiT block forward.  TEST INFRASTRUCTURE ONLY.

This is the plain definition of what the HIP path computes, written with NumPy in float64
so that a reader can check it against the paper by eye.  It is slow on purpose, shares no
code with the HIP library, and may be imported only by the tests, the smoke check and the
benchmark's cpu_baseline leg.  Inputs are the bf16-rounded values the GPU sees, widened
exactly; every later step is float64 with no intermediate rounding, so the oracle is the
exact result the bf16 pipeline approximates.

What is followed:
  * block structure and the operators counted per block: App. B (DiT block; MM-DiT
    double-stream block; MM-DiT single-stream block with its fused linear_1 = QKV + MLP-up
    and fused linear_2 = attention-out + MLP-down);
  * Ulysses sequence parallelism (Sec. 2.1, App. B): the linear layers see this rank's
    N/P tokens, attention sees all N tokens for this rank's H/P heads; the two exchanges
    around attention are replaced by given "peer" tensors (what the other ranks would have
    sent) and by returned "send" tensors (what this rank would have sent);
  * adaLN modulation: xn = LN(x)*(1+scale)+shift and x + gate*branch, with shift/scale/gate
    a plain linear of the timestep embedding; LayerNorm has no affine, biased variance,
    eps 1e-6; q/k RMSNorm is per head over head_dim with a learned weight, eps 1e-6;
    softmax scale 1/sqrt(head_dim), no mask; GELU is the tanh form.  The paper counts these
    operators only as bytes/FLOPs, so these forms are this build's stated reading.

Pinned by tests/test_oracle_*.py (brute-force loops on tiny inputs, softmax row sums,
identity-adaLN collapse, library routines for LayerNorm/GELU/attention special cases, the
P=2 shares reassembling the P=1 block, and MAC counts against the App. B formulas).
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Sequence

import numpy as np
from scipy.special import erf as _erf

LN_EPS = 1e-6
RMS_EPS = 1e-6

KIND_SINGLE, KIND_DIT, KIND_DOUBLE = 0, 1, 2


# ----------------------------------------------------------------------------------------
# storage widening (exact)
# ----------------------------------------------------------------------------------------

def widen(a: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns or any float array -> float64, exactly."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


class MacCounter:
    """Counts multiply-accumulates of the dominant operators, by name (for the App. B pins)."""

    def __init__(self):
        self.macs: Dict[str, int] = {}

    def add(self, name: str, n: int):
        self.macs[name] = self.macs.get(name, 0) + int(n)

    def flops(self, name: Optional[str] = None) -> int:
        if name is None:
            return 2 * sum(self.macs.values())
        return 2 * self.macs.get(name, 0)


# ----------------------------------------------------------------------------------------
# elementary operators
# ----------------------------------------------------------------------------------------

def linear(x: np.ndarray, w: np.ndarray, b: Optional[np.ndarray], mc: Optional[MacCounter] = None,
           name: str = "") -> np.ndarray:
    """y = x @ w^T + b, w stored [out_features, in_features]."""
    y = x @ w.T
    if b is not None:
        y = y + b
    if mc is not None:
        mc.add(name, x.shape[0] * w.shape[0] * w.shape[1])
    return y


def layernorm(x: np.ndarray, eps: float = LN_EPS) -> np.ndarray:
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def modulate(xn: np.ndarray, shift: np.ndarray, scale: np.ndarray) -> np.ndarray:
    return xn * (1.0 + scale) + shift


def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float = RMS_EPS) -> np.ndarray:
    """RMSNorm over the last axis with a learned weight."""
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * w


def rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotary position embedding (not in the paper, which is silent on positions; the models it
    runs rotate q and k): x [n, H, hd]; the pair (x[..., 2i], x[..., 2i+1]) of token row r is
    rotated by the angle whose cosine and sine are cos[r, i], sin[r, i] -- the product of the
    complex number x[2i] + j x[2i+1] with exp(j theta).  The same angles serve every head."""
    a, b = x[..., 0::2], x[..., 1::2]
    c, s_ = cos[:, None, :], sin[:, None, :]
    out = np.empty_like(x)
    out[..., 0::2] = a * c - b * s_
    out[..., 1::2] = a * s_ + b * c
    return out


def _maybe_rope(q, k, inputs, row0=0):
    """q, k [n, H, hd] of local rows row0.. -> rotated when the inputs carry tables."""
    if "rope_cos" not in inputs:
        return q, k
    n = q.shape[0]
    cos = np.asarray(inputs["rope_cos"], dtype=np.float64)[row0:row0 + n]
    sin = np.asarray(inputs["rope_sin"], dtype=np.float64)[row0:row0 + n]
    return rope(q, cos, sin), rope(k, cos, sin)


def gelu_tanh(x: np.ndarray) -> np.ndarray:
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def gelu_erf(x: np.ndarray) -> np.ndarray:
    """GELU proper: x * Phi(x), Phi the standard normal distribution function."""
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def _act(cfg):
    return gelu_erf if getattr(cfg, "gelu_erf", False) else gelu_tanh


def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Two-pass (max-subtracted) softmax over the last axis."""
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, mc: Optional[MacCounter] = None,
              name: str = "attn") -> np.ndarray:
    """Full non-causal softmax attention, brute force.

    q [h, nq, hd], k [h, nk, hd], v [h, nk, hd] -> [h, nq, hd]; the nq x nk score matrix of
    each head is formed in full."""
    h, nq, hd = q.shape
    nk = k.shape[1]
    out = np.empty((h, nq, hd), dtype=np.float64)
    scale = 1.0 / math.sqrt(hd)
    for i in range(h):
        # bounded slabs of query rows: same arithmetic, less memory
        step = max(1, (1 << 26) // max(nk, 1))
        for s in range(0, nq, step):
            p = softmax_rows((q[i, s:s + step] @ k[i].T) * scale)
            out[i, s:s + step] = p @ v[i]
    if mc is not None:
        mc.add(name, 2 * h * nq * nk * hd)
    return out


# ----------------------------------------------------------------------------------------
# Ulysses share bookkeeping
# ----------------------------------------------------------------------------------------

def local_positions(cfg) -> np.ndarray:
    """Positions in the joint sequence of this rank's tokens: contiguous split per stream,
    text rows before image rows in the joint order.  That order is the double-stream block's and,
    in an MMDiT stack (App. B), also that of the single-stream blocks that follow it on the
    concatenated sequence."""
    r, p = cfg.sp_rank, cfg.sp_degree
    if cfg.n_txt > 0:
        tl = cfg.n_txt // p
        il = cfg.n_total // p - tl
        return np.concatenate([np.arange(r * tl, (r + 1) * tl),
                               cfg.n_txt + np.arange(r * il, (r + 1) * il)])
    nl = cfg.n_total // p
    return np.arange(r * nl, (r + 1) * nl)


def joint_attention_share(cfg, q: np.ndarray, k: np.ndarray, v: np.ndarray,
                          peers: Optional[Dict[str, np.ndarray]],
                          rows: Optional[np.ndarray], send_rows: Optional[np.ndarray],
                          mc: Optional[MacCounter]) -> Dict[str, np.ndarray]:
    """The attention stage of one rank.

    q,k,v: [n_local, H, hd] for this rank's tokens and ALL heads (k,v rows needed for every
    local token; q rows are only used at `rows` when row sampling is on).
    Returns
      attn      [len(rows) or n_local, H*hd]  attention output rows for local tokens, all
                heads: this rank's heads computed here, the others taken from peer_attn;
      send_q/k/v [H-H_l, n_local, hd]         what this rank would send (other ranks' heads);
      send_attn [H_l, len(send_rows) or N-n_local, hd]  this rank's heads at remote tokens.
    """
    n_local, H, hd = q.shape
    P, r = cfg.sp_degree, cfg.sp_rank
    hl = H // P
    h0, h1 = r * hl, (r + 1) * hl
    N = cfg.n_total
    lpos = local_positions(cfg)
    out: Dict[str, np.ndarray] = {}

    if P > 1:
        rem = np.ones(N, dtype=bool)
        rem[lpos] = False
        rpos = np.nonzero(rem)[0]
        other = [h for h in range(H) if not (h0 <= h < h1)]
        qsend = q if rows is None else q[np.asarray(rows)]   # sampled: only those rows hold q
        out["send_q"] = np.ascontiguousarray(qsend[:, other].transpose(1, 0, 2))
        out["send_k"] = np.ascontiguousarray(k[:, other].transpose(1, 0, 2))
        out["send_v"] = np.ascontiguousarray(v[:, other].transpose(1, 0, 2))
        K = np.empty((hl, N, hd))
        V = np.empty((hl, N, hd))
        K[:, lpos] = k[:, h0:h1].transpose(1, 0, 2)
        V[:, lpos] = v[:, h0:h1].transpose(1, 0, 2)
        K[:, rpos] = widen(peers["peer_k"])
        V[:, rpos] = widen(peers["peer_v"])
    else:
        rpos = np.zeros(0, dtype=np.int64)
        K = np.ascontiguousarray(k.transpose(1, 0, 2))
        V = np.ascontiguousarray(v.transpose(1, 0, 2))

    sel = np.arange(n_local) if rows is None else np.asarray(rows)
    Ql = np.ascontiguousarray(q[sel][:, h0:h1].transpose(1, 0, 2))        # [hl, n_sel, hd]
    a_loc = attention(Ql, K, V, mc, "attn")                               # [hl, n_sel, hd]
    attn = np.empty((len(sel), H, hd))
    attn[:, h0:h1] = a_loc.transpose(1, 0, 2)
    if P > 1:
        attn[:, other] = widen(peers["peer_attn"])[sel]
        ssel = np.arange(len(rpos)) if send_rows is None else np.asarray(send_rows)
        Qr = widen(peers["peer_q"])[:, ssel]
        out["send_attn"] = attention(Qr, K, V, mc, "attn")
    out["attn"] = attn.reshape(len(sel), H * hd)
    return out


def _split_heads(z: np.ndarray, H: int, hd: int) -> np.ndarray:
    return z.reshape(z.shape[0], H, hd)


# ----------------------------------------------------------------------------------------
# block forwards
# ----------------------------------------------------------------------------------------

def single_stream_block(cfg, params: Dict[str, np.ndarray], inputs: Dict[str, np.ndarray],
                        rows: Optional[Sequence[int]] = None,
                        send_rows: Optional[Sequence[int]] = None,
                        mc: Optional[MacCounter] = None) -> Dict[str, np.ndarray]:
    """MM-DiT single-stream block (App. B), one rank's share.

    With `rows` given, y is produced only for those local token rows (the keys and values
    are still built for every token); `send_rows` likewise samples send_attn."""
    d, H, hd, f = cfg.d, cfg.n_heads, cfg.head_dim, cfg.f
    p = {k_: widen(v_) for k_, v_ in params.items()}
    x = widen(inputs["x"])
    t = widen(inputs["temb"])
    sel = None if rows is None else np.asarray(rows)

    m = p["w_mod"] @ t + p["b_mod"]
    shift, scale, gate = m[:d], m[d:2 * d], m[2 * d:]
    xn = modulate(layernorm(x), shift, scale)

    if sel is None:
        z = linear(xn, p["w1"], p["b1"], mc, "lin1")
        q, k, v, u = z[:, :d], z[:, d:2 * d], z[:, 2 * d:3 * d], z[:, 3 * d:]
        xs = x
    else:
        # keys/values for every local token, queries and MLP-up only at the sampled rows
        kv = linear(xn, p["w1"][d:3 * d], p["b1"][d:3 * d])
        k, v = kv[:, :d], kv[:, d:]
        q = np.zeros_like(k)
        q[sel] = linear(xn[sel], p["w1"][:d], p["b1"][:d])
        u = linear(xn[sel], p["w1"][3 * d:], p["b1"][3 * d:])
        xs = x[sel]
    q, k, v = _split_heads(q, H, hd), _split_heads(k, H, hd), _split_heads(v, H, hd)
    if cfg.qk_rmsnorm:
        q = rmsnorm(q, p["q_norm"])
        k = rmsnorm(k, p["k_norm"])
    q, k = _maybe_rope(q, k, inputs)

    att = joint_attention_share(cfg, q, k, v, inputs, sel, send_rows, mc)
    c = np.concatenate([att["attn"], _act(cfg)(u)], axis=1)
    y = xs + gate * linear(c, p["w2"], p["b2"], mc, "lin2")
    out = {"y": y}
    for key in ("send_q", "send_k", "send_v", "send_attn"):
        if key in att:
            out[key] = att[key]
    return out


def dit_block(cfg, params, inputs, rows=None, send_rows=None, mc=None) -> Dict[str, np.ndarray]:
    """Standard DiT block (App. B): modulated self-attention, cross-attention to the text
    context (pre-norm with affine, no gate, no exchange: the text keys/values are computed
    by every rank), modulated FFN."""
    d, H, hd = cfg.d, cfg.n_heads, cfg.head_dim
    p = {k_: widen(v_) for k_, v_ in params.items()}
    x = widen(inputs["x"])
    t = widen(inputs["temb"])
    ctx = widen(inputs["ctx"])
    sel = None if rows is None else np.asarray(rows)

    m = p["w_mod"] @ t + p["b_mod"]
    sh1, sc1, g1, sh2, sc2, g2 = (m[i * d:(i + 1) * d] for i in range(6))

    h = modulate(layernorm(x), sh1, sc1)
    if sel is None:
        z = linear(h, p["w_qkv"], p["b_qkv"], mc, "self_qkv")
        q, k, v = z[:, :d], z[:, d:2 * d], z[:, 2 * d:]
        xs = x
    else:
        kv = linear(h, p["w_qkv"][d:], p["b_qkv"][d:])
        k, v = kv[:, :d], kv[:, d:]
        q = np.zeros_like(k)
        q[sel] = linear(h[sel], p["w_qkv"][:d], p["b_qkv"][:d])
        xs = x[sel]
    q, k, v = _split_heads(q, H, hd), _split_heads(k, H, hd), _split_heads(v, H, hd)
    if cfg.qk_rmsnorm:
        q = rmsnorm(q, p["q_norm"])
        k = rmsnorm(k, p["k_norm"])
    q, k = _maybe_rope(q, k, inputs)          # self-attention only; the cross-attention below is not rotated
    att = joint_attention_share(cfg, q, k, v, inputs, sel, send_rows, mc)
    x1 = xs + g1 * linear(att["attn"], p["w_o"], p["b_o"], mc, "self_out")

    hc = layernorm(x1) * p["ln_c_w"] + p["ln_c_b"]
    qc = _split_heads(linear(hc, p["w_cq"], p["b_cq"], mc, "cross_q"), H, hd)
    kvc = linear(ctx, p["w_ckv"], p["b_ckv"], mc, "cross_kv")
    kc, vc = _split_heads(kvc[:, :d], H, hd), _split_heads(kvc[:, d:], H, hd)
    if cfg.qk_rmsnorm:
        qc = rmsnorm(qc, p["cq_norm"])
        kc = rmsnorm(kc, p["ck_norm"])
    ac = attention(qc.transpose(1, 0, 2), kc.transpose(1, 0, 2), vc.transpose(1, 0, 2), mc, "cross_attn")
    ac = ac.transpose(1, 0, 2).reshape(x1.shape[0], d)
    x2 = x1 + linear(ac, p["w_co"], p["b_co"], mc, "cross_out")

    h2 = modulate(layernorm(x2), sh2, sc2)
    up = _act(cfg)(linear(h2, p["w_up"], p["b_up"], mc, "ffn_up"))
    y = x2 + g2 * linear(up, p["w_down"], p["b_down"], mc, "ffn_down")
    out = {"y": y}
    for key in ("send_q", "send_k", "send_v", "send_attn"):
        if key in att:
            out[key] = att[key]
    return out


def double_stream_block(cfg, params, inputs, rows=None, send_rows=None, mc=None) -> Dict[str, np.ndarray]:
    """MM-DiT double-stream block (App. B): text and image streams have their own
    modulation, QKV, output projection and FFN; attention is joint over the concatenation
    (text rows, then image rows).  Local rows are ordered text-then-image; `rows` indexes
    that local order.  Returns y (image rows) and y_txt, or y_rows when sampling."""
    d, H, hd = cfg.d, cfg.n_heads, cfg.head_dim
    p = {k_: widen(v_) for k_, v_ in params.items()}
    t = widen(inputs["temb"])
    xs_ = {"txt": widen(inputs["x_txt"]), "img": widen(inputs["x"])}
    tl = xs_["txt"].shape[0]
    nl = tl + xs_["img"].shape[0]
    sel = None if rows is None else np.asarray(rows)

    mod = {}
    qkv = {}
    for s in ("txt", "img"):
        m = p[f"{s}_w_mod"] @ t + p[f"{s}_b_mod"]
        mod[s] = [m[i * d:(i + 1) * d] for i in range(6)]
        h = modulate(layernorm(xs_[s]), mod[s][0], mod[s][1])
        z = linear(h, p[f"{s}_w_qkv"], p[f"{s}_b_qkv"], mc, f"{s}_qkv")
        q, k, v = (_split_heads(z[:, i * d:(i + 1) * d], H, hd) for i in range(3))
        if cfg.qk_rmsnorm:
            q = rmsnorm(q, p[f"{s}_q_norm"])
            k = rmsnorm(k, p[f"{s}_k_norm"])
        q, k = _maybe_rope(q, k, inputs, 0 if s == "txt" else tl)      # table rows: text rows, then image rows
        qkv[s] = (q, k, v)
    q, k, v = (np.concatenate([qkv["txt"][i], qkv["img"][i]], axis=0) for i in range(3))
    att = joint_attention_share(cfg, q, k, v, inputs, sel, send_rows, mc)
    a = att["attn"]                                   # rows: sel or all local (txt then img)
    idx = np.arange(nl) if sel is None else sel

    y_rows = np.empty((len(idx), d))
    for s, mask in (("txt", idx < tl), ("img", idx >= tl)):
        if not mask.any():
            continue
        loc = idx[mask] - (0 if s == "txt" else tl)
        sh1, sc1, g1, sh2, sc2, g2 = mod[s]
        x0 = xs_[s][loc]
        x1 = x0 + g1 * linear(a[mask], p[f"{s}_w_o"], p[f"{s}_b_o"], mc, f"{s}_out")
        h2 = modulate(layernorm(x1), sh2, sc2)
        up = _act(cfg)(linear(h2, p[f"{s}_w_up"], p[f"{s}_b_up"], mc, f"{s}_up"))
        y_rows[mask] = x1 + g2 * linear(up, p[f"{s}_w_down"], p[f"{s}_b_down"], mc, f"{s}_down")
    out = {"y_rows": y_rows}
    if sel is None:
        out["y_txt"], out["y"] = y_rows[:tl], y_rows[tl:]
    for key in ("send_q", "send_k", "send_v", "send_attn"):
        if key in att:
            out[key] = att[key]
    return out


def block_forward(cfg, params, inputs, rows=None, send_rows=None, mc=None):
    fn = {KIND_SINGLE: single_stream_block, KIND_DIT: dit_block, KIND_DOUBLE: double_stream_block}[cfg.kind]
    return fn(cfg, params, inputs, rows, send_rows, mc)
