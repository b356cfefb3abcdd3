"""Element-by-element parity of each HIP kernel against the float64 oracle, through the C ABI."""
import math

import numpy as np
import pytest
import torch

from oracle import block as ob
from oracle import chunks as och
from paper_2605_11335_amd import binding as B
from tests.util import (assert_bf16_close, bf16_round, bits_to_f64, dev_bits, host_bits, max_abs, rel_l2)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_blob(rng, N, K, bias=True, pad_front=512):
    """W [N,K] and bias [N] (bf16) in one byte buffer at 256-aligned offsets."""
    w, wb = bf16_round(rng.normal(size=(N, K)) * 0.05)
    b, bb = bf16_round(rng.normal(size=N) * 0.5)
    w_off = pad_front
    b_off = (w_off + 2 * N * K + 255) // 256 * 256
    buf = np.zeros(b_off + 2 * N + 256, dtype=np.uint8)
    buf[w_off:w_off + 2 * N * K] = wb.reshape(-1).view(np.uint8)
    buf[b_off:b_off + 2 * N] = bb.view(np.uint8)
    return buf, w.astype(np.float64), b.astype(np.float64), w_off, (b_off if bias else -1)


@pytest.mark.parametrize("M,N,K", [(512, 512, 512), (300, 520, 192), (1000, 1304, 256), (2304, 2048, 3072), (37, 8, 64)])
def test_linear_plain(M, N, K):
    rng = np.random.default_rng(M + N + K)
    a, ab = bf16_round(rng.normal(size=(M, K)))
    buf, w, b, w_off, b_off = make_blob(rng, N, K)
    A, blob = dev_bits(ab), torch.from_numpy(buf).to(DEV)
    out = torch.zeros((M, N), dtype=torch.int16, device=DEV)
    B.cf_op_linear(A, blob, w_off, b_off, M, N, K, out)
    torch.cuda.synchronize()
    ref = a.astype(np.float64) @ w.T + b
    assert_bf16_close(host_bits(out), ref, extra_abs=2e-5 * math.sqrt(K))


def test_linear_panels_split_gelu_and_strides():
    """Feature panels launched separately, GELU half into a wider destination, strided A."""
    M, N, K, n_split = 700, 1024, 320, 512
    rng = np.random.default_rng(5)
    lda = K + 64
    a_full, ab = bf16_round(rng.normal(size=(M, lda)))
    a = a_full[:, :K]
    buf, w, b, w_off, b_off = make_blob(rng, N, K)
    A, blob = dev_bits(ab), torch.from_numpy(buf).to(DEV)
    out0 = torch.zeros((M, n_split), dtype=torch.int16, device=DEV)
    ld1 = 104 + (N - n_split)
    out1 = torch.zeros((M, ld1), dtype=torch.int16, device=DEV)
    out1_view = out1[:, 104:]
    for n0, n1 in [(0, 256), (256, 768), (768, 1024)]:
        B.cf_op_linear(A, blob, w_off, b_off, M, N, K, out0, out1_view, n_split=n_split, n0=n0, n1=n1, lda=lda,
                       ld0=n_split, ld1=ld1)
    torch.cuda.synchronize()
    z = a.astype(np.float64) @ w.T + b
    assert_bf16_close(host_bits(out0), z[:, :n_split], extra_abs=1e-4)
    assert_bf16_close(host_bits(out1)[:, 104:], ob.gelu_tanh(z[:, n_split:]), extra_abs=2e-4)
    assert (host_bits(out1)[:, :104] == 0).all()
    # panel decomposition does not change a single bit
    whole = torch.zeros_like(out0)
    whole1 = torch.zeros_like(out1)
    B.cf_op_linear(A, blob, w_off, b_off, M, N, K, whole, whole1[:, 104:], n_split=n_split, lda=lda, ld0=n_split, ld1=ld1)
    torch.cuda.synchronize()
    assert torch.equal(whole, out0) and torch.equal(whole1, out1)


@pytest.mark.parametrize("M,N,K,gate", [(512, 512, 2560, True), (333, 264, 128, False)])
def test_linear_gated_residual(M, N, K, gate):
    rng = np.random.default_rng(9)
    a, ab = bf16_round(rng.normal(size=(M, K)))
    buf, w, b, w_off, b_off = make_blob(rng, N, K)
    resid = rng.normal(size=(M, N)).astype(np.float32)
    g = rng.normal(size=N).astype(np.float32)
    y = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    B.cf_op_linear_residual(dev_bits(ab), torch.from_numpy(buf).to(DEV), w_off, b_off, M, N, K,
                            torch.from_numpy(resid).to(DEV), torch.from_numpy(g).to(DEV) if gate else None, y)
    torch.cuda.synchronize()
    ref = resid.astype(np.float64) + (g.astype(np.float64) if gate else 1.0) * (a.astype(np.float64) @ w.T + b)
    assert max_abs(y.cpu().numpy(), ref) < 5e-5 * math.sqrt(K) and rel_l2(y.cpu().numpy(), ref) < 1e-5


def run_attention(q, k, v, hd):
    H, nq, _ = q.shape
    nk = k.shape[1]
    nk_pad = (nk + 63) // 64 * 64
    _, qb = bf16_round(q)
    _, kb = bf16_round(k)
    _, vb = bf16_round(v)
    vt = np.zeros((H, hd, nk_pad), dtype=np.uint16)
    vt[:, :, :nk] = vb.transpose(0, 2, 1)
    O = torch.zeros((H, nq, hd), dtype=torch.int16, device=DEV)
    B.cf_op_attention(dev_bits(qb), dev_bits(kb), dev_bits(vt), O, H, nq, nk, nk_pad, hd)
    torch.cuda.synchronize()
    ref = ob.attention(bits_to_f64(qb), bits_to_f64(kb), bits_to_f64(vb))
    return bits_to_f64(host_bits(O)), ref


@pytest.mark.parametrize("H,nq,nk,hd,sharp", [(2, 256, 256, 128, 1.0), (3, 200, 333, 128, 1.0), (2, 512, 512, 64, 1.0),
                                              (1, 129, 65, 64, 1.0), (2, 300, 1000, 128, 4.0), (1, 1, 1, 128, 1.0),
                                              (2, 384, 777, 64, 4.0)])
def test_attention(H, nq, nk, hd, sharp):
    rng = np.random.default_rng(H * 1000 + nq + nk + hd)
    q = rng.normal(size=(H, nq, hd)) * sharp
    k = rng.normal(size=(H, nk, hd)) * sharp
    v = rng.normal(size=(H, nk, hd))
    got, ref = run_attention(q, k, v, hd)
    # P is rounded to bf16 before the second contraction and O is stored in bf16
    assert rel_l2(got, ref) < 6e-3, rel_l2(got, ref)
    assert max_abs(got, ref) < 2e-2 * max(1.0, np.abs(ref).max()), max_abs(got, ref)


def test_attention_uniform_values_and_dominant_key():
    rng = np.random.default_rng(77)
    H, n, hd = 1, 200, 128
    q, k = rng.normal(size=(H, n, hd)), rng.normal(size=(H, n, hd))
    v = np.tile(rng.normal(size=(H, 1, hd)), (1, n, 1))
    got, ref = run_attention(q, k, v, hd)
    assert max_abs(got, ref) < 2e-2
    k2 = k.copy()
    k2[0, 150] = q[0, 3] * 50
    v2 = rng.normal(size=(H, n, hd))
    got, ref = run_attention(q, k2, v2, hd)
    assert np.abs(got[0, 3] - bf16_round(v2[0, 150])[0]).max() < 1e-2


@pytest.mark.parametrize("step", [0.7, 3.0, 30.0, 200.0])
def test_attention_scores_that_keep_rising_along_the_keys(step):
    """Every 64-key tile scores `step` nats above the one before it, for every query: whatever reference
    the kernel's online softmax keeps has to move again and again (by a little, by 43 binary orders per
    tile, and by more than exp2 can represent), and late tiles carry nearly all the weight."""
    rng = np.random.default_rng(int(step * 10))
    H, nq, nk, hd = 2, 96, 64 * 9 + 17, 128
    u = rng.normal(size=hd)
    u /= np.linalg.norm(u)
    a = 4.0
    q = a * u + 0.3 * rng.normal(size=(H, nq, hd))
    ramp = (np.arange(nk) // 64) * step * np.sqrt(hd) / a
    k = ramp[None, :, None] * u + 0.3 * rng.normal(size=(H, nk, hd))
    v = rng.normal(size=(H, nk, hd))
    got, ref = run_attention(q, k, v, hd)
    assert np.isfinite(got).all()
    assert rel_l2(got, ref) < 6e-3, rel_l2(got, ref)
    assert max_abs(got, ref) < 2e-2 * max(1.0, np.abs(ref).max()), max_abs(got, ref)


@pytest.mark.parametrize("rows,d", [(100, 512), (37, 3072), (5, 256), (9, 768), (6, 1024), (7, 1536), (3, 2048), (2, 4096)])
def test_ln_modulate(rows, d):
    """Every row width the kernel is built for (d / 256 in 1, 2, 3, 4, 6, 8, 12, 16), row counts that leave
    the last workgroup partly empty."""
    rng = np.random.default_rng(rows + d)
    x = (rng.normal(size=(rows, d)) * 2 + 0.5).astype(np.float32)
    shift, scale = rng.normal(size=d).astype(np.float32), rng.normal(size=d).astype(np.float32)
    out = torch.zeros((rows, d), dtype=torch.int16, device=DEV)
    B.cf_op_ln_modulate(torch.from_numpy(x).to(DEV), torch.from_numpy(shift).to(DEV), torch.from_numpy(scale).to(DEV),
                        out, rows, d)
    torch.cuda.synchronize()
    ref = ob.modulate(ob.layernorm(x.astype(np.float64)), shift.astype(np.float64), scale.astype(np.float64))
    assert_bf16_close(host_bits(out), ref, extra_abs=1e-5)


@pytest.mark.parametrize("n,K", [(1536, 512), (70, 1024), (264, 2560), (96, 4096), (50, 768), (33, 3072)])
def test_modvec(n, K):
    """One, two, three and four steps of the walk over K per trip (K = 2560 ends on a trip whose last steps
    lie past the row, K = 768 on a step only half the lanes take part in); row counts that are not whole waves."""
    rng = np.random.default_rng(3 + n + K)
    buf, w, b, w_off, b_off = make_blob(rng, n, K)
    t = rng.normal(size=K).astype(np.float32)
    m = torch.zeros(n, dtype=torch.float32, device=DEV)
    B.cf_op_modvec(torch.from_numpy(buf).to(DEV), w_off, b_off, torch.from_numpy(t).to(DEV), m, n, K)
    torch.cuda.synchronize()
    ref = w @ t.astype(np.float64) + b
    assert max_abs(m.cpu().numpy(), ref) < 1e-4


@pytest.mark.parametrize("nbytes,first", [(8, 0), (4096, 17), (1 << 20, 12345), (8 * 1001, 3)])
def test_checksum_bit_exact(nbytes, first):
    rng = np.random.default_rng(nbytes)
    data = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
    got = B.cf_op_checksum(torch.from_numpy(data).to(DEV), nbytes, first)
    assert got == och.checksum_words(data, first)


def test_launch_checks_reject_bad_shapes():
    z = torch.zeros(1024, dtype=torch.int16, device=DEV)
    with pytest.raises(B.ChunkflowError):
        B.cf_op_linear(z, z, 0, -1, 4, 8, 48, z)          # K not a multiple of 64
    with pytest.raises(B.ChunkflowError):
        B.cf_op_linear(z, z, 0, -1, 4, 12, 64, z)         # N not a multiple of 8
    with pytest.raises(B.ChunkflowError):
        B.cf_op_attention(z, z, z, z, 1, 4, 4, 4, 128)    # nk_pad not a multiple of 64
    with pytest.raises(B.ChunkflowError):
        B.cf_op_attention(z, z, z, z, 1, 4, 4, 64, 96)    # head_dim


@pytest.mark.parametrize("M,N,K", [(1, 8, 64), (257, 264, 64), (3, 4096, 128), (4097, 16, 192)])
def test_linear_degenerate_shapes(M, N, K):
    rng = np.random.default_rng(M * 7 + N + K)
    a, ab = bf16_round(rng.normal(size=(M, K)))
    buf, w, b, w_off, b_off = make_blob(rng, N, K)
    out = torch.zeros((M, N), dtype=torch.int16, device=DEV)
    B.cf_op_linear(dev_bits(ab), torch.from_numpy(buf).to(DEV), w_off, b_off, M, N, K, out)
    torch.cuda.synchronize()
    assert_bf16_close(host_bits(out), a.astype(np.float64) @ w.T + b, extra_abs=1e-4)


@pytest.mark.parametrize("H,nq,nk,hd", [(1, 5, 64, 128), (1, 130, 129, 128), (2, 1, 4097, 64), (1, 4100, 3, 128)])
def test_attention_ragged_extremes(H, nq, nk, hd):
    rng = np.random.default_rng(nq * 13 + nk)
    got, ref = run_attention(rng.normal(size=(H, nq, hd)), rng.normal(size=(H, nk, hd)), rng.normal(size=(H, nk, hd)), hd)
    assert rel_l2(got, ref) < 6e-3 and max_abs(got, ref) < 2e-2 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("H,n,hd", [(12, 4608, 128), (8, 5000, 64), (16, 4608, 128), (16, 4608, 64), (4, 12800, 128)])
def test_attention_every_workgroup_height(H, n, hd):
    """Shapes whose grids make the launcher pick 8, 8 (ragged), 4, 4 and 7 waves per workgroup."""
    rng = np.random.default_rng(H + n + hd)
    got, ref = run_attention(rng.normal(size=(H, n, hd)), rng.normal(size=(H, n, hd)), rng.normal(size=(H, n, hd)), hd)
    assert rel_l2(got, ref) < 6e-3 and max_abs(got, ref) < 2e-2 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("H,n,hd,step", [(12, 4608, 128, 3.0), (12, 4608, 128, 200.0), (8, 5000, 64, 200.0), (4, 12800, 128, 30.0),
                                         (4, 12800, 128, 200.0)])
def test_attention_rising_scores_at_every_workgroup_height(H, n, hd, step):
    """The first ten key tiles score `step` nats above one another (then the level holds) on grids that run 8, 8 (ragged,
    64-wide heads) and 7 waves per workgroup: the softmax reference is shifted tile after tile (3 and 30 nats) or the
    workgroups repeat their sweep (200 nats)."""
    rng = np.random.default_rng(int(H + n + hd + step))
    u = rng.normal(size=hd)
    u /= np.linalg.norm(u)
    a = 4.0
    q = a * u + 0.3 * rng.normal(size=(H, n, hd))
    ramp = np.minimum(np.arange(n) // 64, 9) * step * np.sqrt(hd) / a
    k = ramp[None, :, None] * u + 0.3 * rng.normal(size=(H, n, hd))
    got, ref = run_attention(q, k, rng.normal(size=(H, n, hd)), hd)
    assert np.isfinite(got).all()
    assert rel_l2(got, ref) < 6e-3 and max_abs(got, ref) < 2e-2 * max(1.0, np.abs(ref).max())


def test_linear_under_one_round_of_tiles():
    """A grid that covers the chip less than once (both epilogues), with a ragged feature edge."""
    rng = np.random.default_rng(21)
    M, N, K = 2304, 3080, 256
    a, ab = bf16_round(rng.normal(size=(M, K)))
    buf, w, b, w_off, b_off = make_blob(rng, N, K)
    blob = torch.from_numpy(buf).to(DEV)
    out = torch.zeros((M, N), dtype=torch.int16, device=DEV)
    B.cf_op_linear(dev_bits(ab), blob, w_off, b_off, M, N, K, out)
    resid = rng.normal(size=(M, N)).astype(np.float32)
    g = rng.normal(size=N).astype(np.float32)
    y = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    B.cf_op_linear_residual(dev_bits(ab), blob, w_off, b_off, M, N, K, torch.from_numpy(resid).to(DEV),
                            torch.from_numpy(g).to(DEV), y)
    torch.cuda.synchronize()
    z = a.astype(np.float64) @ w.T + b
    assert_bf16_close(host_bits(out), z, extra_abs=1e-4)
    assert max_abs(y.cpu().numpy(), resid + g.astype(np.float64) * z) < 1e-3


@pytest.mark.parametrize("M,N", [(2304, 4096), (2100, 2056)])
def test_linear_every_epilogue_on_both_tiles(M, N):
    """The first shape fills the chip better with 256 x 256 tiles, the second (ragged in both directions)
    with 128 x 128 ones; each runs the split epilogue with either activation and the gated residual one."""
    K, n_split = 192, 1024
    rng = np.random.default_rng(M + N)
    a, ab = bf16_round(rng.normal(size=(M, K)))
    buf, w, b, w_off, b_off = make_blob(rng, N, K)
    A, blob = dev_bits(ab), torch.from_numpy(buf).to(DEV)
    z = a.astype(np.float64) @ w.T + b
    for erf_form in (False, True):
        out0 = torch.zeros((M, n_split), dtype=torch.int16, device=DEV)
        out1 = torch.zeros((M, N - n_split), dtype=torch.int16, device=DEV)
        B.cf_op_linear(A, blob, w_off, b_off, M, N, K, out0, out1, n_split=n_split, gelu_erf=erf_form)
        torch.cuda.synchronize()
        act = ob.gelu_erf if erf_form else ob.gelu_tanh
        assert_bf16_close(host_bits(out0), z[:, :n_split], extra_abs=1e-4)
        assert_bf16_close(host_bits(out1), act(z[:, n_split:]), extra_abs=2e-4)
    resid = rng.normal(size=(M, N)).astype(np.float32)
    g = rng.normal(size=N).astype(np.float32)
    y = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    B.cf_op_linear_residual(A, blob, w_off, b_off, M, N, K, torch.from_numpy(resid).to(DEV), torch.from_numpy(g).to(DEV), y)
    torch.cuda.synchronize()
    assert max_abs(y.cpu().numpy(), resid + g.astype(np.float64) * z) < 1e-3


def test_linear_gelu_forms_are_told_apart():
    """The epilogue's two activations (tanh form, erf form) against the oracle's: pre-activations
    are spread over +-6 so that the region where the forms differ by several bf16 ulps (around
    -2.5, where GELU itself is small) is populated; each output matches its own reference and
    not the other's."""
    M, N, K = 512, 512, 320
    rng = np.random.default_rng(11)
    a, ab = bf16_round(rng.normal(size=(M, K)))
    w, wb = bf16_round(rng.normal(size=(N, K)) * 0.12)
    buf = np.zeros(2 * N * K + 256, dtype=np.uint8)
    buf[:2 * N * K] = wb.reshape(-1).view(np.uint8)
    A, blob = dev_bits(ab), torch.from_numpy(buf).to(DEV)
    z = a.astype(np.float64) @ w.astype(np.float64).T
    outs = {}
    for erf_form in (False, True):
        out = torch.zeros((M, N), dtype=torch.int16, device=DEV)
        B.cf_op_linear(A, blob, 0, -1, M, N, K, None, out, n_split=0, gelu_erf=erf_form)
        torch.cuda.synchronize()
        outs[erf_form] = bits_to_f64(host_bits(out))
    refs = {False: ob.gelu_tanh(z), True: ob.gelu_erf(z)}
    tol = lambda ref: 2.0 ** -8 * np.abs(ref) * 2 + 6e-5
    for form in (False, True):
        assert (np.abs(outs[form] - refs[form]) <= tol(refs[form])).all(), form
        assert (np.abs(outs[form] - refs[not form]) > tol(refs[not form])).sum() > 100, form


def test_mfma_rate_diagnostic_runs_and_is_deterministic():
    out = torch.zeros(256 * 256, dtype=torch.float32, device=DEV)
    res = []
    for rnd in (False, True, True):
        B.cf_op_mfma_rate(50, rnd, out)
        torch.cuda.synchronize()
        res.append(out.cpu().numpy().copy())
        assert np.isfinite(res[-1]).all() and np.abs(res[-1]).max() > 0
    assert np.array_equal(res[1], res[2]) and not np.array_equal(res[0], res[1])
    with pytest.raises(B.ChunkflowError):
        B.cf_op_mfma_rate(0, False, out)


def test_mix_rate_diagnostic_runs_for_every_built_mix_and_rejects_others():
    out = torch.zeros(256 * 512, dtype=torch.float32, device=DEV)
    ref = None
    for waves, reads, valu, exps in [(4, 0, 0, 0), (8, 0, 0, 0), (8, 16, 0, 0), (8, 8, 0, 0), (8, 0, 4, 1), (8, 16, 4, 1), (4, 8, 2, 1)]:
        out.zero_()
        B.cf_op_mix_rate(20, waves, reads, valu, exps, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()[:256 * 64 * waves]
        assert np.isfinite(got).all() and np.abs(got).max() > 0, (waves, reads, valu, exps)
        if (waves, reads, valu, exps) == (8, 0, 0, 0):
            ref = got.copy()
    B.cf_op_mix_rate(20, 8, 0, 0, 0, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy()[:256 * 64 * 8], ref)         # deterministic
    for bad in [(0, 8, 0, 0, 0), (20, 5, 0, 0, 0), (20, 8, 3, 0, 0), (20, 8, 16, 4, 0)]:
        with pytest.raises(B.ChunkflowError):
            B.cf_op_mix_rate(*bad, out)
