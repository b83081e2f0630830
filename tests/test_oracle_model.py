"""Pins for the checker's forward/backward and optimizer steps (Appendix A, Sections 3.4 and 4.1)."""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle import model, move, optim
from oracle.sample import KIND_FFN, KIND_HEAD, sample_plan

GPT = si.ModelCfg(n_layers=2, d_model=16, n_heads=4, d_head=4, d_ff=24, vocab=13, max_seq=8)
LLAMA = si.ModelCfg(arch="llama", n_layers=2, d_model=16, n_heads=4, d_head=4, d_ff=24, vocab=13, max_seq=8,
                    act="swiglu", norm="rms", has_bias=False, tied_head=False, rope=True)
BLOCK = si.ModelCfg(n_layers=1, d_model=16, n_heads=4, d_head=4, d_ff=24, vocab=0, max_seq=8)
BLOCK_LLAMA = replace(LLAMA, vocab=0, n_layers=1)
# ReLU is the activation of the paper's analysis (Appendix A.1, FFN definition); GELU and SwiGLU are the workloads'
CASES = {"gpt": GPT, "llama": LLAMA, "block": BLOCK, "block_llama": BLOCK_LLAMA, "gpt_relu": replace(GPT, act="relu"),
         "block_relu": replace(BLOCK, act="relu")}


def _data(cfg, B=2, N=6, seed=1):
    if cfg.vocab:
        t = si.tokens_uniform(cfg.vocab, B, N, seed)
        return t[:, :-1], t[:, 1:]
    return si.activations(cfg, B, N, seed, "x"), si.activations(cfg, B, N, seed, "y")


# ------------------------------------------------------------------ independent library graph
def _torch_forward(cfg, P, inputs, targets, c_scale):
    """The same model, phrased with library building blocks only (layer_norm, SDPA, gelu, cross_entropy,
    complex-number rotary), so that agreement is not a re-typing of the checker's formulas."""
    G = P["globals"]
    if cfg.vocab:
        tok = torch.as_tensor(np.asarray(inputs), dtype=torch.long)
        X = F.embedding(tok, G["tok_embed"])
        B, N = tok.shape
        if "pos_embed" in G:
            X = X + G["pos_embed"][:N]
    else:
        X = torch.as_tensor(inputs)
        B, N, _ = X.shape
    d, dh = cfg.d_model, cfg.d_head

    def norm(x, w, b):
        if cfg.norm == "ln":
            return F.layer_norm(x, (d,), w, b, cfg.norm_eps)
        return F.rms_norm(x, (d,), w, cfg.norm_eps)

    def rope(x):  # x [B,H,N,dh]; pair (i, i+dh/2) as one complex number
        half = dh // 2
        z = torch.complex(x[..., :half], x[..., half:])
        freqs = torch.arange(N, dtype=torch.float64)[:, None] / (cfg.rope_theta ** (2 * torch.arange(half, dtype=torch.float64) / dh))[None, :]
        z = z * torch.polar(torch.ones_like(freqs), freqs)
        return torch.cat([z.real, z.imag], -1)

    for lw, (c_a, c_f) in zip(P["layers"], c_scale):
        Hs = lw["wq"].shape[0] // dh
        h = norm(X, lw["norm1_w"], lw.get("norm1_b"))
        q, k, v = (F.linear(h, lw["w" + n], lw.get("b" + n)).view(B, N, Hs, dh).transpose(1, 2) for n in "qkv")
        if cfg.rope:
            q, k = rope(q), rope(k)
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(B, N, Hs * dh)
        X = X + c_a * F.linear(o, lw["wo"], lw.get("bo"))
        h = norm(X, lw["norm2_w"], lw.get("norm2_b"))
        u = F.linear(h, lw["w_up"], lw.get("b_up"))
        if cfg.act == "swiglu":
            a = F.silu(F.linear(h, lw["w_gate"])) * u
        elif cfg.act == "relu":
            a = F.relu(u)
        else:
            a = F.gelu(u, approximate="tanh")
        X = X + c_f * F.linear(a, lw["w_down"], lw.get("b_down"))
    if cfg.vocab:
        hf = norm(X, G["final_norm_w"], G.get("final_norm_b"))
        logits = F.linear(hf, G["tok_embed"] if cfg.tied_head else G["lm_head"])
        return F.cross_entropy(logits.view(B * N, -1), torch.as_tensor(np.asarray(targets), dtype=torch.long).view(-1))
    return F.mse_loss(X, torch.as_tensor(targets))


def _to_torch(P):
    return {"layers": [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in lw.items()} for lw in P["layers"]],
            "globals": {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in P["globals"].items()}}


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("sub", [False, True])
def test_matches_library_graph_and_autograd(name, sub):
    cfg = CASES[name]
    P = si.make_weights(cfg, 3, std=0.4, generic=True)
    if sub:   # a half-width subnet, scaled
        plan = sample_plan(cfg.n_layers, 4, cfg.n_ffn_units, 2, 2, cfg.n_ffn_units // 2, seed=2)
        P = move.extract(P, plan, 1, cfg.d_head)
    x, y = _data(cfg)
    loss, grads = model.forward_backward(cfg, P, x, y, scale_mode=True)
    Pt = _to_torch(P)
    cs = [model.scale_factors(cfg, lw, True) for lw in P["layers"]]
    if sub:
        assert cs[0] == (math.sqrt(2.0), math.sqrt(2.0))
    lt = _torch_forward(cfg, Pt, x, y, cs)
    assert abs(loss - lt.item()) < 1e-12 * max(1, abs(loss))
    lt.backward()
    for l, lw in enumerate(Pt["layers"]):
        for k, t in lw.items():
            np.testing.assert_allclose(grads["layers"][l][k], t.grad.numpy(), rtol=1e-9, atol=1e-13, err_msg=f"L{l}.{k}")
    for k, t in Pt["globals"].items():
        np.testing.assert_allclose(grads["globals"][k], t.grad.numpy(), rtol=1e-9, atol=1e-13, err_msg=k)


@pytest.mark.parametrize("name", list(CASES))
def test_central_finite_differences(name):
    cfg = CASES[name]
    P = si.make_weights(cfg, 5, std=0.4, generic=True)
    plan = sample_plan(cfg.n_layers, 4, cfg.n_ffn_units, 2, 3, 16, seed=2)
    P = move.extract(P, plan, 0, cfg.d_head)
    x, y = _data(cfg, seed=4)
    _, grads = model.forward_backward(cfg, P, x, y)
    rng = np.random.default_rng(0)
    eps = 1e-6

    def check(arr, g, tag):
        for _ in range(3):
            pos = tuple(rng.integers(0, n) for n in arr.shape)
            old = arr[pos]
            arr[pos] = old + eps
            lp = model.forward_loss(cfg, P, x, y)
            arr[pos] = old - eps
            lm_ = model.forward_loss(cfg, P, x, y)
            arr[pos] = old
            fd = (lp - lm_) / (2 * eps)
            assert abs(fd - g[pos]) < 1e-7 * max(1.0, abs(fd)) + 2e-9, (tag, pos, fd, g[pos])

    for l, lw in enumerate(P["layers"]):
        for k, a in lw.items():
            check(a, grads["layers"][l][k], f"L{l}.{k}")
    for k, a in P["globals"].items():
        check(a, grads["globals"][k], k)
    if not cfg.vocab:   # gradient with respect to the input activations
        check(x, grads["input"], "input")


# ------------------------------------------------------------------ masked equivalence (Section 4.1)
def _masked_full(cfg, full, plan, s):
    """Masked TwIST: the full model with the inactive heads' and neurons' parameters zeroed."""
    M = {"layers": [], "globals": full["globals"]}
    for l, lw in enumerate(full["layers"]):
        out = {}
        for name, w in lw.items():
            if name in move.PARTITIONED:
                kind, axis = move.PARTITIONED[name]
                qb = cfg.d_head if kind == KIND_HEAD else cfg.ffn_granule
                keep = np.zeros(w.shape[axis], bool)
                keep[move.element_index(plan[l][kind]["idx"][s], qb)] = True
                out[name] = w * (keep[:, None] if (axis == 0 and w.ndim == 2) else keep)
            else:
                out[name] = w
        M["layers"].append(out)
    return M


@pytest.mark.parametrize("name", ["gpt", "llama", "block"])
@pytest.mark.parametrize("scale_mode", [False, True])
def test_subnet_equals_masked_full_model(name, scale_mode, monkeypatch):
    cfg = CASES[name]
    full = si.make_weights(cfg, 7, std=0.4, generic=True)
    S = 2
    plan = sample_plan(cfg.n_layers, 4, cfg.n_ffn_units, S, 2, cfg.n_ffn_units // 2, seed=6)
    x, y = _data(cfg, seed=8)
    for s in range(S):
        sub = move.extract(full, plan, s, cfg.d_head)
        loss_s, g_s, out_s = model.forward_backward(cfg, sub, x, y, scale_mode=scale_mode, return_out=True)
        masked = _masked_full(cfg, full, plan, s)
        # the masked model applies the same constant as the subnet (Masked TwIST keeps the scaling hooks)
        consts = [model.scale_factors(cfg, lw, scale_mode) for lw in sub["layers"]]
        it = iter(consts * 2)
        monkeypatch.setattr(model, "scale_factors", lambda *_a, **_k: next(it))
        loss_m, g_m, out_m = model.forward_backward(cfg, masked, x, y, scale_mode=scale_mode, return_out=True)
        monkeypatch.undo()
        np.testing.assert_allclose(out_s, out_m, rtol=1e-12, atol=1e-13)
        assert abs(loss_s - loss_m) < 1e-13 * max(1, abs(loss_m))
        # gradient flow: gradients of the kept blocks agree, shared ones agree
        g_keep = move.extract({"layers": g_m["layers"], "globals": g_m["globals"]}, plan, s, cfg.d_head)
        for l in range(cfg.n_layers):
            for k in g_s["layers"][l]:
                np.testing.assert_allclose(g_s["layers"][l][k], g_keep["layers"][l][k], rtol=1e-10, atol=1e-14, err_msg=k)
        for k in g_s["globals"]:
            np.testing.assert_allclose(g_s["globals"][k], g_m["globals"][k], rtol=1e-10, atol=1e-14)


def test_full_width_subnet_is_unscaled_full_model():
    cfg = GPT
    full = si.make_weights(cfg, 9, std=0.4, generic=True)
    plan = sample_plan(cfg.n_layers, 4, cfg.n_ffn_units, 2, 4, cfg.n_ffn_units, seed=1)
    sub = move.extract(full, plan, 1, cfg.d_head)
    x, y = _data(cfg)
    assert model.forward_loss(cfg, sub, x, y, True) == model.forward_loss(cfg, full, x, y, False)


# ------------------------------------------------------------------ the rounding hook
@pytest.mark.parametrize("name", ["gpt", "llama", "block_relu"])
def test_rounding_hook_is_inert_by_default_and_sees_exactly_the_declared_tensor_classes(name):
    """The optional hook q(tag, array) is where the bf16 parity tests snap tensors to the bf16 grid.  Pinned here:
    (a) a hook that returns its argument leaves loss and every gradient bit-identical to the plain call, so the hook
    adds no arithmetic of its own; (b) the tensor classes it is offered are exactly the declared list, so a new
    rounding point cannot appear without this test (and the tolerance derivation that counts these points) changing;
    (c) the number of offers per layer is fixed; (d) a hook that does round changes the result (it is not ignored)."""
    cfg = CASES[name]
    P = si.make_weights(cfg, 11, std=0.4, generic=True)
    x, y = _data(cfg, seed=3)
    seen = []

    def spy(tag, a):
        seen.append(tag)
        return a

    plain = model.forward_backward(cfg, P, x, y)
    hooked = model.forward_backward(cfg, P, x, y, q=spy)
    assert plain[0] == hooked[0]
    for l in range(cfg.n_layers):
        for k, g in plain[1]["layers"][l].items():
            assert np.array_equal(g, hooked[1]["layers"][l][k]), (l, k)
    for k, g in plain[1]["globals"].items():
        assert np.array_equal(g, hooked[1]["globals"][k]), k
    assert model.HOOK_TAGS == ("h1", "qkv", "p", "o", "h2", "u", "a", "hf", "logits", "dlogits", "dres", "dact", "ds")
    lm_tags = {"hf", "logits", "dlogits"}
    assert set(seen) == set(model.HOOK_TAGS) - (set() if cfg.vocab else lm_tags)
    # offers per layer, forward: h1, q, k, v (+ rotated q, k), the probabilities, o, h2, u (+ gate), a; backward: dres x 2,
    # the gradient of a, of u (+ gate), of h2, of o, the probabilities again (value gradient), the score gradient, the
    # gradients of q, k, v (+ the two rounding points before the inverse rotation), of h1
    rope, gated = int(cfg.rope), int(cfg.act == "swiglu")
    fwd = 9 + 2 * rope + gated
    bwd = 2 + 1 + 1 + gated + 1 + 1 + 2 + 3 + 2 * rope + 1
    head = 2 + 2 if cfg.vocab else 0          # hf, logits; dlogits, the gradient of hf
    assert len(seen) == cfg.n_layers * (fwd + bwd) + head, (len(seen), fwd, bwd, head)
    rounded = model.forward_backward(cfg, P, x, y, q=lambda tag, a: si.to_bf16_grid(a))
    assert rounded[0] != plain[0] and abs(rounded[0] - plain[0]) < 0.05 * abs(plain[0])


def test_standalone_pieces_against_library_routines():
    """The pieces the per-kernel GPU tests call one by one, each against a library routine or its autograd."""
    rng = np.random.default_rng(5)
    g, u, da = rng.standard_normal((3, 7, 12))
    tg, tu = (torch.tensor(a, requires_grad=True) for a in (g, u))
    ta = F.silu(tg) * tu
    np.testing.assert_allclose(model.swiglu_fwd(g, u), ta.detach().numpy(), rtol=1e-13)
    ta.backward(torch.tensor(da))
    dg, du = model.swiglu_bwd(g, u, da)
    np.testing.assert_allclose(dg, tg.grad.numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(du, tu.grad.numpy(), rtol=1e-12, atol=1e-15)
    for kind, fn in (("relu", F.relu), ("gelu_tanh", lambda t: F.gelu(t, approximate="tanh"))):
        t = torch.tensor(u, requires_grad=True)
        out = fn(t)
        np.testing.assert_allclose(model.act_fwd(u, kind), out.detach().numpy(), rtol=1e-13, atol=1e-16)
        out.backward(torch.tensor(da))
        np.testing.assert_allclose(da * model.act_bwd(u, kind), t.grad.numpy(), rtol=1e-12, atol=1e-15)
    logits = rng.standard_normal((2, 5, 9)) * 3
    tgt = rng.integers(0, 9, (2, 5))
    tl = torch.tensor(logits, requires_grad=True)
    lt = F.cross_entropy(tl.view(10, 9), torch.tensor(tgt).view(-1))
    lt.backward()
    loss, dl = model.cross_entropy(logits, tgt)
    assert abs(loss - lt.item()) < 1e-14
    np.testing.assert_allclose(dl, tl.grad.numpy(), rtol=1e-12, atol=1e-16)
    for kind, lib in (("ln", lambda t, w, b: F.layer_norm(t, (12,), w, b, 1e-5)), ("rms", lambda t, w, b: F.rms_norm(t, (12,), w, 1e-5))):
        x, w, b, dy = rng.standard_normal((7, 12)), rng.standard_normal(12), rng.standard_normal(12), rng.standard_normal((7, 12))
        tx, tw, tb = (torch.tensor(a, requires_grad=True) for a in (x, w, b))
        ty = lib(tx, tw, tb)
        yv, cache = model.norm_fwd(x, w, b if kind == "ln" else None, kind, 1e-5)
        np.testing.assert_allclose(yv, ty.detach().numpy(), rtol=1e-12, atol=1e-15)
        ty.backward(torch.tensor(dy))
        dx, dw, db = model.norm_bwd(dy, w, cache, kind)
        np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(dw, tw.grad.numpy(), rtol=1e-11, atol=1e-14)
        if kind == "ln":
            np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-11, atol=1e-14)
    tok = rng.integers(0, 6, (2, 4))
    E, Pz, dX = rng.standard_normal((6, 3)), rng.standard_normal((5, 3)), rng.standard_normal((2, 4, 3))
    tE, tP = torch.tensor(E, requires_grad=True), torch.tensor(Pz, requires_grad=True)
    tX = F.embedding(torch.tensor(tok), tE) + tP[:4]
    np.testing.assert_allclose(model.embed_fwd(tok, E, Pz), tX.detach().numpy(), rtol=1e-15)
    tX.backward(torch.tensor(dX))
    dE = np.zeros_like(E)
    dP = model.embed_bwd(tok, dX, dE, 5)
    np.testing.assert_allclose(dE, tE.grad.numpy(), rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(dP, tP.grad.numpy(), rtol=1e-13, atol=1e-16)
    # rotary: a rotation of each (i, i + d_head/2) pair by pos * theta^(-2i/d_head) = multiplication of the complex number
    x = rng.standard_normal((1, 5, 2, 8))
    cos, sin = model.rope_tables(5, 8, 100.0)
    z = (x[..., :4] + 1j * x[..., 4:]) * np.exp(1j * np.arange(5)[:, None] * 100.0 ** (-2.0 * np.arange(4) / 8))[None, :, None, :]
    np.testing.assert_allclose(model.rope_apply(x, cos, sin), np.concatenate([z.real, z.imag], -1), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(model.rope_apply(model.rope_apply(x, cos, sin), cos, sin, -1.0), x, rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------------ scale-factor theorems (Appendix A.3)
def test_monte_carlo_scale_factors():
    """At the initialisation of Appendix A.3, dropping FFN neurons (ReLU) scales E||y||^2 by d'/d
    (Theorem A.3) and dropping heads scales it by H'/H (Theorem A.7); after the sqrt(N_full/N_sub)
    correction of Section 3.4 both ratios are 1.  Also Var([y_ffn]_i) = 1 (Lemma A.5)."""
    d, H, dh, Fi, N, B = 64, 8, 8, 256, 16, 8
    cfg = si.ModelCfg(n_layers=1, d_model=d, n_heads=H, d_head=dh, d_ff=Fi, vocab=0, act="relu", has_bias=False, max_seq=N)
    acc = {"ffn_full": 0.0, "ffn_sub": 0.0, "attn_full": 0.0, "attn_sub": 0.0}
    trials = 40
    for t in range(trials):
        P = {"globals": {}, "layers": [{
            "wq": si.normal(t, "q", (H * dh, d), d ** -0.5), "wk": si.normal(t, "k", (H * dh, d), d ** -0.5),
            "wv": si.normal(t, "v", (H * dh, d), d ** -0.5), "wo": si.normal(t, "o", (d, H * dh), (H * dh) ** -0.5),
            "w_up": si.normal(t, "u", (Fi, d), (2.0 / d) ** 0.5), "w_down": si.normal(t, "dn", (d, Fi), Fi ** -0.5),
            "norm1_w": np.ones(d), "norm1_b": np.zeros(d), "norm2_w": np.ones(d), "norm2_b": np.zeros(d)}]}
        plan = sample_plan(1, H, Fi, 2, H // 2, Fi // 2, seed=t)
        sub = move.extract(P, plan, 0, dh)
        X = si.normal(t, "x", (B, N, d))
        for tag, W in (("full", P), ("sub", sub)):
            lw = W["layers"][0]
            zero_ffn = {"layers": [dict(lw, w_down=np.zeros_like(lw["w_down"]))], "globals": {}}
            zero_att = {"layers": [dict(lw, wo=np.zeros_like(lw["wo"]))], "globals": {}}
            # module outputs = block output minus its input, with the other module silenced, unscaled
            ya = model.forward_backward(cfg, zero_ffn, X, X, scale_mode=False, need_grads=False, return_out=True)[2] - X
            yf = model.forward_backward(cfg, zero_att, X, X, scale_mode=False, need_grads=False, return_out=True)[2] - X
            acc["attn_" + tag] += (ya ** 2).sum() / trials
            acc["ffn_" + tag] += (yf ** 2).sum() / trials
            if tag == "full":
                var_ffn = (yf ** 2).mean()
    assert abs(acc["ffn_sub"] / acc["ffn_full"] - 0.5) < 0.02
    assert abs(acc["attn_sub"] / acc["attn_full"] - 0.5) < 0.03
    assert abs(var_ffn - 1.0) < 0.1
    c_a, c_f = model.scale_factors(cfg, sub["layers"][0], True)
    assert abs(c_a ** 2 * acc["attn_sub"] / acc["attn_full"] - 1.0) < 0.06
    assert abs(c_f ** 2 * acc["ffn_sub"] / acc["ffn_full"] - 1.0) < 0.04


# ------------------------------------------------------------------ optimizer closed forms
def test_sgd_and_adamw_scalar_closed_form():
    P = {"layers": [{"w": np.array([[2.0]]), "b": np.array([1.0])}], "globals": {}}
    G = {"layers": [{"w": np.array([[0.5]]), "b": np.array([-0.25])}], "globals": {}}
    optim.sgd_step(P, G, 0.1)
    assert P["layers"][0]["w"][0, 0] == 2.0 - 0.05 and P["layers"][0]["b"][0] == 1.0 + 0.025
    # AdamW with a constant gradient: mhat = g, vhat = g^2 at every step, so each step moves by
    # lr*(sign(g)/(1+eps/|g|) + wd*w) for the matrix and lr*sign(g)/(1+eps/|g|) for the vector.
    P = {"layers": [{"w": np.array([[2.0]]), "b": np.array([1.0])}], "globals": {}}
    st = optim.adamw_init(P)
    w, b = 2.0, 1.0
    lr, wd, eps = 1e-2, 0.1, 1e-8
    for _ in range(3):
        optim.adamw_step(P, G, st, lr=lr, eps=eps, weight_decay=wd)
        w = w - lr * (0.5 / (0.5 + eps) + wd * w)
        b = b - lr * (-0.25 / (0.25 + eps))
        assert abs(P["layers"][0]["w"][0, 0] - w) < 1e-15 and abs(P["layers"][0]["b"][0] - b) < 1e-15
    # a changing gradient, against the unrolled textbook recurrences
    gs = [0.3, -0.7, 0.2]
    P = {"layers": [{"b": np.array([0.0])}], "globals": {}}
    st = optim.adamw_init(P)
    m = v = 0.0
    x = 0.0
    for t, g in enumerate(gs, 1):
        optim.adamw_step(P, {"layers": [{"b": np.array([g])}], "globals": {}}, st, lr=0.1)
        m = 0.9 * m + 0.1 * g
        v = 0.999 * v + 0.001 * g * g
        x -= 0.1 * (m / (1 - 0.9 ** t)) / (math.sqrt(v / (1 - 0.999 ** t)) + 1e-8)
        assert abs(P["layers"][0]["b"][0] - x) < 1e-15
