"""Kernel-level parity of the memory-bound steps of the subnet pass (norms, rotary positions, activations, loss,
embedding, the Masked-TwIST masks), each against the checker's unrounded fp64 function on identical inputs:
<= 5e-3 where a bf16 result is stored (one rounding: about 1.1e-3), <= 1e-4 for fp32 results of either model type."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as si
from helpers import rel_fro, to_numpy
from oracle import model as omodel

pytestmark = pytest.mark.gpu

BF, F32 = "bf16", "f32"


def _snap(a, dtype):
    return si.to_bf16_grid(a) if dtype == BF else np.asarray(a, np.float32).astype(np.float64)


def _dev(a, dtype=None):
    t = torch.tensor(np.ascontiguousarray(a), dtype=torch.float64)
    return t.to({BF: torch.bfloat16, F32: torch.float32, None: torch.float32}[dtype]).cuda().contiguous()


def _tol(dtype):
    return 5e-3 if dtype == BF else 1e-4


# d_model: 256, 768, 2048, 4096 take the kernels that hold a row in registers (1, 3, 8, 16 vectors per lane), 200 the
# general kernels; T = 37 leaves a ragged last chunk of 16 rows
@pytest.mark.parametrize("dtype", [BF, F32])
@pytest.mark.parametrize("kind,D,T", [("rms", 256, 37), ("ln", 256, 64), ("ln", 768, 37), ("rms", 2048, 50), ("rms", 4096, 33), ("ln", 200, 37),
                                       ("rms", 200, 16), ("ln", 1024, 19)])
def test_norm_forward_and_backward(lib, dtype, kind, D, T):
    cfg = si.ModelCfg(d_model=D, n_heads=1, d_head=8, d_ff=8, norm=kind, dtype=dtype)
    ctx = lib.Context(lib.desc_from_cfg(cfg))
    x = np.asarray(si.normal(D + T, "x", (T, D), 1.5) + 0.3, np.float32).astype(np.float64)      # the residual stream is fp32
    w, b = _snap(1.0 + si.normal(D, "w", (D,), 0.2), dtype), _snap(si.normal(D, "b", (D,), 0.2), dtype)
    dy = _snap(si.normal(T, "dy", (T, D)), dtype)
    bb = b if kind == "ln" else None
    y, stats, (dx, dxb, dw, db) = ctx.twist_norm_raw(_dev(x), _dev(w, dtype), _dev(bb, dtype) if bb is not None else None, _dev(dy, dtype))
    torch.cuda.synchronize()
    want_y, cache = omodel.norm_fwd(x, w, bb, kind, cfg.norm_eps)
    want_dx, want_dw, want_db = omodel.norm_bwd(dy, w, cache, kind)
    assert rel_fro(to_numpy(y), want_y) <= _tol(dtype)
    np.testing.assert_allclose(to_numpy(stats[:, 1]), cache[1][:, 0], rtol=1e-5)
    assert rel_fro(to_numpy(dx), want_dx) <= 1e-4                      # fp32 result in both model types
    assert rel_fro(to_numpy(dxb), want_dx) <= _tol(dtype)
    assert rel_fro(to_numpy(dw), want_dw) <= 1e-4
    if kind == "ln":
        assert rel_fro(to_numpy(db), want_db) <= 1e-4


@pytest.mark.parametrize("dtype", [BF, F32])
@pytest.mark.parametrize("dh,Hs,B,N", [(128, 2, 2, 48), (64, 3, 1, 40), (6, 5, 2, 9)])
def test_rotary_positions(lib, dtype, dh, Hs, B, N):
    cfg = si.ModelCfg(arch="llama", d_model=64, n_heads=Hs, d_head=dh, d_ff=8, rope=True, dtype=dtype)
    ctx = lib.Context(lib.desc_from_cfg(cfg))
    qkv = _snap(si.normal(dh, "qkv", (B * N, 3 * Hs * dh)), dtype)
    cos, sin = omodel.rope_tables(N, dh, cfg.rope_theta)
    for sign in (1.0, -1.0):
        t = _dev(qkv, dtype)
        ctx.twist_rope_raw(t, B, N, Hs, sign)
        torch.cuda.synchronize()
        got = to_numpy(t)
        heads = qkv.reshape(B, N, 3 * Hs, dh)
        want = heads.copy()
        want[:, :, :2 * Hs] = omodel.rope_apply(heads[:, :, :2 * Hs], cos, sin, sign)       # q and k heads turn, v stays
        assert rel_fro(got, want.reshape(B * N, -1)) <= _tol(dtype)
        assert np.array_equal(got.reshape(B, N, 3 * Hs, dh)[:, :, 2 * Hs:], heads[:, :, 2 * Hs:])


@pytest.mark.parametrize("dtype", [BF, F32])
@pytest.mark.parametrize("act,T,F,unit", [("swiglu", 37, 352, 1), ("swiglu", 5, 44, 4), ("gelu_tanh", 37, 512, 1), ("gelu_tanh", 9, 35, 5),
                                           ("relu", 37, 512, 64), ("relu", 9, 35, 7), ("relu", 3, 12, 1)])
def test_activation_forward_backward_and_neuron_mask(lib, dtype, act, T, F, unit):
    """Without a mask: a = f(u), dgu = da f'(u).  With the Masked-TwIST mask (Section 4.1, y = M * f(x)): masked blocks give
    exact zeros in a and dgu, kept blocks the unmasked values bit for bit."""
    cfg = si.ModelCfg(d_model=64, n_heads=1, d_head=8, d_ff=F, ffn_granule=unit, act=act, has_bias=act != "swiglu", dtype=dtype)
    ctx = lib.Context(lib.desc_from_cfg(cfg))
    nf = 2 if act == "swiglu" else 1
    gu = _snap(si.normal(F, "gu", (T, nf * F), 1.5), dtype)
    da = _snap(si.normal(T, "da", (T, F)), dtype)
    a, dgu = ctx.twist_act_raw(_dev(gu, dtype), F, _dev(da, dtype))
    torch.cuda.synchronize()
    if act == "swiglu":
        g, u = gu[:, :F], gu[:, F:]
        want_a = omodel.swiglu_fwd(g, u)
        dg, du = omodel.swiglu_bwd(g, u, da)
        want_d = np.concatenate([dg, du], axis=1)
    else:
        want_a, want_d = omodel.act_fwd(gu, act), da * omodel.act_bwd(gu, act)
    assert rel_fro(to_numpy(a), want_a) <= _tol(dtype), rel_fro(to_numpy(a), want_a)
    assert rel_fro(to_numpy(dgu), want_d) <= _tol(dtype), rel_fro(to_numpy(dgu), want_d)
    rng = np.random.default_rng(F + unit)
    keep_np = np.where(rng.random(F // unit) < 0.5, -1, rng.integers(0, 100, F // unit)).astype(np.int32)
    keep_np[0], keep_np[-1] = -1, 3
    keep = torch.tensor(keep_np).cuda()
    am, dm = ctx.twist_act_raw(_dev(gu, dtype), F, _dev(da, dtype), keep=keep, unit=unit)
    torch.cuda.synchronize()
    on = np.repeat(keep_np >= 0, unit)
    am, dm, a, dgu = (to_numpy(t) for t in (am, dm, a, dgu))
    assert not am[:, ~on].any() and np.array_equal(am[:, on], a[:, on])
    on2 = np.tile(on, nf)
    assert not dm[:, ~on2].any() and np.array_equal(dm[:, on2], dgu[:, on2])


# vocabulary: 515 and 1003 (rows held in registers, 4 vectors per lane), 32000 (16 vectors), 33001 (re-read kernel); the
# row stride is the vocabulary rounded up to 8, as in the training pass; 301 with fp32 takes the general kernel
@pytest.mark.parametrize("dtype,V,T", [(BF, 515, 37), (BF, 1003, 8), (BF, 32000, 6), (BF, 33001, 5), (F32, 301, 37), (F32, 1003, 5)])
def test_cross_entropy_loss_and_gradient(lib, dtype, V, T):
    cfg = si.ModelCfg(d_model=64, n_heads=1, d_head=8, d_ff=8, vocab=V, dtype=dtype)
    ctx = lib.Context(lib.desc_from_cfg(cfg))
    ld = (V + 7) // 8 * 8
    logits = _snap(si.normal(V, "logits", (T, V), 2.0), dtype)
    tgt = si.tokens_uniform(V, 1, T - 1, V)[0].astype(np.int32)
    tgt[0], tgt[-1] = V - 1, 0
    padded = np.full((T, ld), 7.0)                                        # the padding must not enter the sums
    padded[:, :V] = logits
    t = _dev(padded, dtype)
    loss, rowloss = ctx.twist_ce_raw(t, torch.tensor(tgt).cuda())
    torch.cuda.synchronize()
    want_loss, want_d = omodel.cross_entropy(logits[None], tgt[None].astype(np.int64))
    assert abs(loss.item() - want_loss) <= 1e-5 * abs(want_loss), (loss.item(), want_loss)
    got = to_numpy(t)
    assert rel_fro(got[:, :V], want_d[0]) <= _tol(dtype), rel_fro(got[:, :V], want_d[0])
    if dtype == BF:
        assert not got[:, V:].any()                                       # padding columns feed the next projection as zeros
    np.testing.assert_allclose(to_numpy(rowloss).mean(), want_loss, rtol=1e-5)


@pytest.mark.parametrize("dtype", [BF, F32])
@pytest.mark.parametrize("positions", [True, False])
def test_embedding_forward_and_backward(lib, dtype, positions):
    V, D, B, N, P = 53, 72, 3, 10, 12
    cfg = si.ModelCfg(d_model=D, n_heads=1, d_head=8, d_ff=8, vocab=V, max_seq=P, dtype=dtype)
    ctx = lib.Context(lib.desc_from_cfg(cfg))
    E, Pz = _snap(si.normal(1, "E", (V, D)), dtype), _snap(si.normal(2, "P", (P, D)), dtype)
    tok = si.tokens_uniform(V, B, N - 1, 5).astype(np.int32)
    tok[0, :3] = 7                                                          # a repeated token: its gradient rows add up
    dx = np.asarray(si.normal(3, "dx", (B, N, D)), np.float32).astype(np.float64)
    x, d_tok, d_pos = ctx.twist_embed_raw(torch.tensor(tok).cuda(), _dev(E, dtype), _dev(Pz, dtype) if positions else None, _dev(dx.reshape(B * N, D)))
    torch.cuda.synchronize()
    want_x = omodel.embed_fwd(tok.astype(np.int64), E, Pz if positions else None)
    assert rel_fro(to_numpy(x), want_x.reshape(B * N, D)) <= 1e-6          # exact: a copy and at most one fp32 add
    dE = np.zeros((V, D))
    dP = omodel.embed_bwd(tok.astype(np.int64), dx, dE, P if positions else None)
    assert rel_fro(to_numpy(d_tok), dE) <= 1e-6
    if positions:
        assert rel_fro(to_numpy(d_pos), dP[:N]) <= 1e-6


@pytest.mark.parametrize("dtype,dh,N,choice", [(BF, 128, 256, {}), (BF, 128, 128, {"staged_attention": True}), (BF, 64, 128, {}),
                                               (BF, 32, 40, {}), (BF, 128, 128, {"plain_only": True}), (F32, 16, 37, {}),
                                               # one, three and five key blocks: the dK/dV kernel pairs key blocks, the middle one stays single
                                               (BF, 128, 128, {}), (BF, 128, 384, {}), (BF, 128, 640, {})])
def test_attention_head_mask(lib, dtype, dh, N, choice):
    """Masked TwIST's head mask inside the attention kernels (Section 4.1): a masked head's output and its q, k, v gradients
    are exact zeros, the kept heads' results are bit-identical to the unmasked call, in every kernel family (direct-to-LDS,
    register-staged, plain)."""
    Hs, B = 4, 2
    cfg = si.ModelCfg(d_model=64, n_heads=Hs, d_head=dh, d_ff=8, dtype=dtype, max_seq=N)
    ctx = lib.Context(lib.desc_from_cfg(cfg))
    ctx.twist_set_kernel_choice(**choice)
    qkv = _dev(_snap(si.normal(dh + N, "qkv", (B * N, 3 * Hs * dh)), dtype), dtype)
    dout = _dev(_snap(si.normal(N, "dout", (B * N, Hs * dh)), dtype), dtype)
    o, lse, dqkv = ctx.twist_attention_raw(qkv, dout, B, N, Hs)
    keep_np = np.array([5, -1, 0, -1], np.int32)
    om, lsem, dm = ctx.twist_attention_raw(qkv, dout, B, N, Hs, keep=torch.tensor(keep_np).cuda())
    torch.cuda.synchronize()
    o, om = to_numpy(o).reshape(B * N, Hs, dh), to_numpy(om).reshape(B * N, Hs, dh)
    d, dm = to_numpy(dqkv).reshape(B * N, 3, Hs, dh), to_numpy(dm).reshape(B * N, 3, Hs, dh)
    on = keep_np >= 0
    assert not om[:, ~on].any() and not dm[:, :, ~on].any()
    assert np.array_equal(om[:, on], o[:, on]) and np.array_equal(dm[:, :, on], d[:, :, on])
    assert o[:, ~on].any() and d[:, :, ~on].any()
    # and the unmasked results are the checker's attention (forward and backward) on the same inputs
    q, k, v = (to_numpy(qkv).reshape(B, N, 3, Hs, dh)[:, :, i] for i in range(3))
    want_o, p = omodel.attention_fwd(q, k, v)
    assert rel_fro(o.reshape(B, N, Hs, dh), want_o) <= _tol(dtype)
    wdq, wdk, wdv = omodel.attention_bwd(p, q, k, v, to_numpy(dout).reshape(B, N, Hs, dh))
    for i, want in enumerate((wdq, wdk, wdv)):
        assert rel_fro(d[:, i].reshape(B, N, Hs, dh), want) <= _tol(dtype), (i, rel_fro(d[:, i].reshape(B, N, Hs, dh), want))


@pytest.mark.parametrize("dh,N,choice", [(128, 256, {}), (128, 384, {}), (128, 128, {"staged_attention": True}), (64, 128, {}), (32, 40, {})])
def test_attention_backward_through_rotary_positions(lib, dh, N, choice):
    """The q and k gradients turned back through the rotary embedding (inside the direct-to-LDS kernels, by a separate
    rotation behind the others): the checker's attention backward followed by the inverse rotation."""
    Hs, B = 2, 2
    cfg = si.ModelCfg(arch="llama", d_model=64, n_heads=Hs, d_head=dh, d_ff=8, rope=True, dtype=BF, max_seq=N)
    ctx = lib.Context(lib.desc_from_cfg(cfg))
    ctx.twist_set_kernel_choice(**choice)
    qkv = _dev(_snap(si.normal(dh, "qkv", (B * N, 3 * Hs * dh)), BF), BF)
    dout = _dev(_snap(si.normal(N, "dout", (B * N, Hs * dh)), BF), BF)
    o, lse, dqkv = ctx.twist_attention_raw(qkv, dout, B, N, Hs, rope_backward=True)
    torch.cuda.synchronize()
    q, k, v = (to_numpy(qkv).reshape(B, N, 3, Hs, dh)[:, :, i] for i in range(3))
    _, p = omodel.attention_fwd(q, k, v)
    dq, dk, dv = omodel.attention_bwd(p, q, k, v, to_numpy(dout).reshape(B, N, Hs, dh))
    cos, sin = omodel.rope_tables(N, dh, cfg.rope_theta)
    want = (omodel.rope_apply(dq, cos, sin, -1.0), omodel.rope_apply(dk, cos, sin, -1.0), dv)
    got = to_numpy(dqkv).reshape(B, N, 3, Hs, dh)
    for i in range(3):
        assert rel_fro(got[:, :, i], want[i]) <= 5e-3, (i, rel_fro(got[:, :, i], want[i]))
