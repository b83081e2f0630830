"""Dense pre-norm transformer of a given (possibly reduced) width: loss and all parameter gradients.

Test infrastructure (see the package docstring).  fp64 numpy, one plain step after another.

Forward (Appendix A.1-A.2 in the paper's notation, [out,in] weight storage):
  per layer   X_ln  = f_ln(X)
              head_h = softmax(Q_h K_h^T / sqrt(d_head) + causal mask) V_h,   Q_h = X_ln W^Q_h (+ b) ...
              Y_attn = Concat(head_1..head_H') C^attn (+ b)
              X     <- X + c_attn * Y_attn                     c_attn = sqrt(H / H')    (Section 3.4)
              X_ln2 = f_ln(X)
              Y_ffn = C^ffn sigma(W^ffn X_ln2 (+ b)) (+ b)      or  C^ffn (silu(W^gate x) * W^ffn x)
              X     <- X + c_ffn * Y_ffn                       c_ffn = sqrt(U / U')
  language-model mode: X_0 = token embedding (+ learned positions), final norm, projection to the
  vocabulary (tied to the token embedding for GPT), mean next-token cross-entropy over B*N positions.
  block-stack mode (vocab = 0): X_0 is given, the loss is the mean squared error over B*N*d.

The scale multiplies the whole module output (projection and its bias) right before the residual
add and is differentiated through as a constant; a full-width module has factor 1, which is the
"no scaling, no masking" full-model evaluation rule of Section 4.2.

Backward: the analytic gradient of exactly this graph, written out by hand.

`q` is an optional rounding hook q(tag, array) -> array, identity by default.  The bf16 parity tests
pass one that snaps named tensors to the bf16 grid, to follow the precision the paper leaves unstated.
"""
import math

import numpy as np


def _ident(tag, a):
    return a


# Every tensor class the rounding hook is offered, i.e. every place where a bf16 model stores an activation or an
# activation gradient between two kernels: normed inputs (h1, h2, hf), projections of them (qkv, also after the rotary
# embedding; u: FFN pre-activations, gate included), attention output (o), FFN activation (a), logits; backward: the
# loss gradient (dlogits), the residual-stream gradient handed to a module (dres) and every activation gradient (dact);
# and the two tensors a tiled attention kernel hands to the matrix cores in bf16 without ever storing them: the
# probabilities (p, forward and in the value gradient) and the score gradient (ds).
HOOK_TAGS = ("h1", "qkv", "p", "o", "h2", "u", "a", "hf", "logits", "dlogits", "dres", "dact", "ds")


# ----------------------------------------------------------------------------- pieces
def norm_fwd(x, w, b, kind, eps):
    if kind == "ln":
        mu = x.mean(-1, keepdims=True)
        var = ((x - mu) ** 2).mean(-1, keepdims=True)
        rstd = 1.0 / np.sqrt(var + eps)
        z = (x - mu) * rstd
    else:  # rms
        rstd = 1.0 / np.sqrt((x ** 2).mean(-1, keepdims=True) + eps)
        z = x * rstd
    y = z * w + (b if b is not None else 0.0)
    return y, (z, rstd)


def norm_bwd(dy, w, cache, kind):
    z, rstd = cache
    dz = dy * w
    dw = (dy * z).reshape(-1, z.shape[-1]).sum(0)
    db = dy.reshape(-1, z.shape[-1]).sum(0)
    if kind == "ln":
        dx = rstd * (dz - dz.mean(-1, keepdims=True) - z * (dz * z).mean(-1, keepdims=True))
    else:
        dx = rstd * (dz - z * (dz * z).mean(-1, keepdims=True))
    return dx, dw, db


_K0 = math.sqrt(2.0 / math.pi)
_K1 = 0.044715


def act_fwd(u, kind):
    if kind == "relu":
        return np.maximum(u, 0.0)
    if kind == "gelu_tanh":
        return 0.5 * u * (1.0 + np.tanh(_K0 * (u + _K1 * u ** 3)))
    raise ValueError(kind)


def act_bwd(u, kind):
    if kind == "relu":
        return (u > 0).astype(u.dtype)
    t = np.tanh(_K0 * (u + _K1 * u ** 3))
    return 0.5 * (1.0 + t) + 0.5 * u * (1.0 - t * t) * _K0 * (1.0 + 3.0 * _K1 * u * u)


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def swiglu_fwd(g, u):
    """Gated FFN activation: silu(g) * u with silu(g) = g * sigmoid(g)."""
    return g * sigmoid(g) * u


def swiglu_bwd(g, u, da):
    """(dg, du) of swiglu_fwd given the gradient da of its output."""
    sg = sigmoid(g)
    return da * u * (sg + g * sg * (1.0 - sg)), da * g * sg


def cross_entropy(logits, tgt):
    """Mean next-token cross-entropy over all leading positions of logits [..., V] with integer targets [...], and
    its gradient with respect to the logits, (softmax - onehot) / #positions."""
    m = logits.max(-1, keepdims=True)
    lse = m[..., 0] + np.log(np.exp(logits - m).sum(-1))
    picked = np.take_along_axis(logits, tgt[..., None], axis=-1)[..., 0]
    loss = float((lse - picked).mean())
    dlogits = np.exp(logits - lse[..., None])
    np.put_along_axis(dlogits, tgt[..., None], np.take_along_axis(dlogits, tgt[..., None], -1) - 1.0, -1)
    return loss, dlogits / lse.size


def embed_fwd(tok, tok_embed, pos_embed=None):
    """X_0 [B, N, d]: the token's embedding row plus (GPT) the learned embedding of its position."""
    X = tok_embed[tok]
    if pos_embed is not None:
        X = X + pos_embed[None, :tok.shape[1], :]
    return X


def embed_bwd(tok, dX, d_tok_embed, n_pos=None):
    """Adds dX [B, N, d] into the rows of d_tok_embed the batch used (in place); returns the gradient of the position
    table [n_pos, d] (rows beyond N zero) when n_pos is given."""
    B, N, _ = dX.shape
    np.add.at(d_tok_embed, tok.reshape(-1), dX.reshape(B * N, -1))
    if n_pos is None:
        return None
    dP = np.zeros((n_pos, dX.shape[-1]))
    dP[:N] = dX.sum(0)
    return dP


def rope_tables(N, d_head, theta):
    half = d_head // 2
    inv_freq = theta ** (-2.0 * np.arange(half) / d_head)
    ang = np.arange(N)[:, None] * inv_freq[None, :]
    return np.cos(ang), np.sin(ang)                      # [N, half]


def rope_apply(x, cos, sin, sign=1.0):
    """x [B, N, H, d_head]; pair (i, i + d_head/2) rotated by sign * pos * theta^(-2i/d_head)."""
    half = x.shape[-1] // 2
    a, b = x[..., :half], x[..., half:]
    c, s = cos[None, :, None, :], sign * sin[None, :, None, :]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


# ----------------------------------------------------------------------------- model
def attention_fwd(qh, kh, vh, q=_ident):
    """Causal multi-head attention of Appendix A.1 on [B, N, H, d_head] arrays: softmax(Q K^T / sqrt(d_head)) V
    per head with keys after the query masked out.  Returns (output [B, N, H, d_head], probabilities [B, H, N, N]).
    A rounding hook is offered the probabilities ("p"); rounded probabilities are renormalised to sum to one, so that
    the output stays a convex combination of the value rows (what a kernel that feeds rounded probabilities to the
    matrix cores and divides by their sum computes)."""
    N, dh = qh.shape[1], qh.shape[3]
    causal = np.triu(np.ones((N, N), dtype=bool), k=1)
    sc = np.einsum("bnhe,bmhe->bhnm", qh, kh) / math.sqrt(dh)
    sc = np.where(causal[None, None], -np.inf, sc)
    sc = sc - sc.max(-1, keepdims=True)
    p = np.exp(sc)
    p = p / p.sum(-1, keepdims=True)
    pr = q("p", p)
    if pr is not p:
        p = pr / pr.sum(-1, keepdims=True)
    return np.einsum("bhnm,bmhe->bnhe", p, vh), p


def attention_bwd(p, qh, kh, vh, do, q=_ident):
    """Gradients of attention_fwd's output with respect to q, k, v given d(output) = do (all [B, N, H, d_head]).
    A rounding hook is offered the probabilities where they enter the value gradient ("p") and the score gradient
    where it enters the query and key gradients ("ds")."""
    dh = qh.shape[3]
    dv = np.einsum("bhnm,bnhe->bmhe", q("p", p), do)
    dp = np.einsum("bnhe,bmhe->bhnm", do, vh)
    ds = q("ds", p * (dp - (dp * p).sum(-1, keepdims=True)) / math.sqrt(dh))
    dq = np.einsum("bhnm,bmhe->bnhe", ds, kh)
    dk = np.einsum("bhnm,bnhe->bmhe", ds, qh)
    return dq, dk, dv


def scale_factors(cfg, lw, scale_mode):
    """(c_attn, c_ffn) of one layer, from the subnet's widths."""
    if not scale_mode:
        return 1.0, 1.0
    h_sub = lw["wq"].shape[0] // cfg.d_head
    u_sub = lw["w_up"].shape[0] // cfg.ffn_granule
    return math.sqrt(cfg.n_heads / h_sub), math.sqrt(cfg.n_ffn_units / u_sub)


def forward_backward(cfg, P, inputs, targets, scale_mode=True, q=_ident, need_grads=True, return_out=False):
    """loss, grads (same nesting as P).  inputs: int tokens [B,N] or activations [B,N,d]."""
    dh = cfg.d_head
    G = P["globals"]
    lm = cfg.vocab > 0
    if lm:
        tok = np.asarray(inputs)
        B, N = tok.shape
        X = embed_fwd(tok, G["tok_embed"], G.get("pos_embed"))
    else:
        X = np.asarray(inputs, dtype=np.float64)
        B, N, _ = X.shape
    cos, sin = rope_tables(N, dh, cfg.rope_theta) if cfg.rope else (None, None)
    caches = []

    for lw in P["layers"]:
        c_a, c_f = scale_factors(cfg, lw, scale_mode)
        Hs = lw["wq"].shape[0] // dh
        c = {"X0": X}
        h, c["n1"] = norm_fwd(X, lw["norm1_w"], lw.get("norm1_b"), cfg.norm, cfg.norm_eps)
        h = q("h1", h)
        c["h"] = h
        qh = h @ lw["wq"].T + lw.get("bq", 0.0)
        kh = h @ lw["wk"].T + lw.get("bk", 0.0)
        vh = h @ lw["wv"].T + lw.get("bv", 0.0)
        qh, kh, vh = (q("qkv", t).reshape(B, N, Hs, dh) for t in (qh, kh, vh))
        if cfg.rope:
            qh, kh = q("qkv", rope_apply(qh, cos, sin)), q("qkv", rope_apply(kh, cos, sin))
        o, p = attention_fwd(qh, kh, vh, q)
        o = q("o", o.reshape(B, N, Hs * dh))
        c.update(q=qh, k=kh, v=vh, p=p, o=o)
        y = o @ lw["wo"].T + lw.get("bo", 0.0)
        X = X + c_a * y
        c["X1"] = X
        h2, c["n2"] = norm_fwd(X, lw["norm2_w"], lw.get("norm2_b"), cfg.norm, cfg.norm_eps)
        h2 = q("h2", h2)
        c["h2"] = h2
        u = q("u", h2 @ lw["w_up"].T + lw.get("b_up", 0.0))
        c["u"] = u
        if cfg.act == "swiglu":
            g = q("u", h2 @ lw["w_gate"].T)
            c["g"] = g
            a = swiglu_fwd(g, u)
        else:
            a = act_fwd(u, cfg.act)
        a = q("a", a)
        c["a"] = a
        y2 = a @ lw["w_down"].T + lw.get("b_down", 0.0)
        X = X + c_f * y2
        caches.append(c)

    if lm:
        hf, nf = norm_fwd(X, G["final_norm_w"], G.get("final_norm_b"), cfg.norm, cfg.norm_eps)
        hf = q("hf", hf)
        W_out = G["tok_embed"] if cfg.tied_head else G["lm_head"]
        logits = q("logits", hf @ W_out.T)                                    # [B,N,V]
        tgt = np.asarray(targets)
        loss, dlogits = cross_entropy(logits, tgt)
    else:
        Y = np.asarray(targets, dtype=np.float64)
        loss = float(((X - Y) ** 2).mean())
    if not need_grads:
        return (loss, None, X) if return_out else (loss, None)

    # ------------------------------------------------------------------ backward
    grads = {"layers": [None] * len(P["layers"]), "globals": {}}
    if lm:
        dlogits = q("dlogits", dlogits)
        dW_out = dlogits.reshape(B * N, -1).T @ hf.reshape(B * N, -1)
        dhf = q("dact", dlogits @ W_out)
        dX, dw, db = norm_bwd(dhf, G["final_norm_w"], nf, cfg.norm)
        grads["globals"]["final_norm_w"] = dw
        if "final_norm_b" in G:
            grads["globals"]["final_norm_b"] = db
        if cfg.tied_head:
            grads["globals"]["tok_embed"] = dW_out
        else:
            grads["globals"]["lm_head"] = dW_out
            grads["globals"]["tok_embed"] = np.zeros_like(G["tok_embed"])
    else:
        dX = 2.0 * (X - Y) / X.size

    for li in range(len(P["layers"]) - 1, -1, -1):
        lw, c = P["layers"][li], caches[li]
        c_a, c_f = scale_factors(cfg, lw, scale_mode)
        Hs = lw["wq"].shape[0] // dh
        T = B * N
        g_ = {}
        # FFN branch
        dy2 = q("dres", dX) * c_f
        dy2f = dy2.reshape(T, -1)
        g_["w_down"] = dy2f.T @ c["a"].reshape(T, -1)
        if "b_down" in lw:
            g_["b_down"] = dy2f.sum(0)
        da = q("dact", dy2 @ lw["w_down"])
        if cfg.act == "swiglu":
            dg, du = swiglu_bwd(c["g"], c["u"], da)
            dg, du = q("dact", dg), q("dact", du)
            g_["w_gate"] = dg.reshape(T, -1).T @ c["h2"].reshape(T, -1)
            dh2 = dg @ lw["w_gate"]
        else:
            du = q("dact", da * act_bwd(c["u"], cfg.act))
            dh2 = 0.0
        g_["w_up"] = du.reshape(T, -1).T @ c["h2"].reshape(T, -1)
        if "b_up" in lw:
            g_["b_up"] = du.reshape(T, -1).sum(0)
        dh2 = q("dact", dh2 + du @ lw["w_up"])
        dxn, g_["norm2_w"], db = norm_bwd(dh2, lw["norm2_w"], c["n2"], cfg.norm)
        if "norm2_b" in lw:
            g_["norm2_b"] = db
        dX = dX + dxn
        # attention branch
        dy = q("dres", dX) * c_a
        dyf = dy.reshape(T, -1)
        g_["wo"] = dyf.T @ c["o"].reshape(T, -1)
        if "bo" in lw:
            g_["bo"] = dyf.sum(0)
        do = q("dact", dy @ lw["wo"]).reshape(B, N, Hs, dh)
        p, qh, kh, vh = c["p"], c["q"], c["k"], c["v"]
        dq, dk, dv = attention_bwd(p, qh, kh, vh, do, q)
        if cfg.rope:
            dq, dk = q("dact", dq), q("dact", dk)      # rounding point only; identity by default
            dq, dk = rope_apply(dq, cos, sin, -1.0), rope_apply(dk, cos, sin, -1.0)
        dq, dk, dv = (q("dact", t).reshape(T, Hs * dh) for t in (dq, dk, dv))
        hf_ = c["h"].reshape(T, -1)
        g_["wq"], g_["wk"], g_["wv"] = dq.T @ hf_, dk.T @ hf_, dv.T @ hf_
        if "bq" in lw:
            g_["bq"], g_["bk"], g_["bv"] = dq.sum(0), dk.sum(0), dv.sum(0)
        dh1 = q("dact", (dq @ lw["wq"] + dk @ lw["wk"] + dv @ lw["wv"]).reshape(B, N, -1))
        dxn, g_["norm1_w"], db = norm_bwd(dh1, lw["norm1_w"], c["n1"], cfg.norm)
        if "norm1_b" in lw:
            g_["norm1_b"] = db
        dX = dX + dxn
        grads["layers"][li] = g_

    if lm:
        dP = embed_bwd(tok, dX, grads["globals"]["tok_embed"], G["pos_embed"].shape[0] if "pos_embed" in G else None)
        if dP is not None:
            grads["globals"]["pos_embed"] = dP
    else:
        grads["input"] = dX
    return (loss, grads, X) if return_out else (loss, grads)


def forward_loss(cfg, P, inputs, targets, scale_mode=True):
    return forward_backward(cfg, P, inputs, targets, scale_mode, need_grads=False)[0]
