"""Local optimizer steps on a subnet's parameters, fp64.

Test infrastructure (see the package docstring).  The paper trains with Adam at lr 1e-4
(Section 5, "Setup"); the workloads here use plain SGD for the fp32 block and AdamW with
decoupled weight decay for the Llama-shaped one.  Decay touches matrices only.

  SGD    w <- w - lr g
  AdamW  m <- b1 m + (1-b1) g ;  v <- b2 v + (1-b2) g^2
         w <- w - lr ( (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps) + wd w )
"""
import numpy as np


def _walk(P):
    for l, lw in enumerate(P["layers"]):
        for k in lw:
            yield ("layers", l, k)
    for k in P["globals"]:
        yield ("globals", None, k)


def _get(T, key):
    a, l, k = key
    return T[a][l][k] if a == "layers" else T[a][k]


def _set(T, key, v):
    a, l, k = key
    if a == "layers":
        T[a][l][k] = v
    else:
        T[a][k] = v


def sgd_step(P, grads, lr):
    for key in _walk(P):
        _set(P, key, _get(P, key) - lr * _get(grads, key))


def adamw_init(P):
    z = {"t": 0, "m": {"layers": [dict() for _ in P["layers"]], "globals": {}},
         "v": {"layers": [dict() for _ in P["layers"]], "globals": {}}}
    for key in _walk(P):
        _set(z["m"], key, np.zeros_like(_get(P, key)))
        _set(z["v"], key, np.zeros_like(_get(P, key)))
    return z


def adamw_step(P, grads, state, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    state["t"] += 1
    t = state["t"]
    for key in _walk(P):
        w, g = _get(P, key), _get(grads, key)
        m = beta1 * _get(state["m"], key) + (1 - beta1) * g
        v = beta2 * _get(state["v"], key) + (1 - beta2) * g * g
        _set(state["m"], key, m)
        _set(state["v"], key, v)
        mhat = m / (1 - beta1 ** t)
        vhat = v / (1 - beta2 ** t)
        wd = weight_decay if w.ndim == 2 else 0.0
        _set(P, key, w - lr * (mhat / (np.sqrt(vhat) + eps) + wd * w))
