"""Dispatcher (extract) and aggregator, as plain definitions in fp64.

Test infrastructure (see the package docstring).

extract  (Section 3.2): a partitioned tensor is cut into blocks along its block axis and the
         blocks a blueprint row names are concatenated in that order; shared tensors are copied.
aggregate (Section 3.3): p <- sum_i p_i [p in W_i] / sum_i [p in W_i].  The p on the right is read
         as subnet i's trained copy.  A parameter no subnet holds keeps its central value
         (Figure 3's caption calls such parameters frozen).  Shared parameters sit in every
         subnet, so their rule is the plain mean over the S subnets.

Block structure (Section 3.1): an attention block is one head = d_head rows of W^Q, W^K, W^V
(and of their biases) plus d_head columns of C^attn; an FFN block is `granule` rows of W^ffn
(and of its bias, and of the gate matrix in gated FFNs) plus `granule` columns of C^ffn.
Matrices are stored [out_features, in_features].  The output biases of C^attn and C^ffn, the
norms, the embeddings and the final projection are shared (Appendix C counts them unscaled).
"""
import numpy as np

from .sample import KIND_FFN, KIND_HEAD

# name -> (kind, block axis)
PARTITIONED = {
    "wq": (KIND_HEAD, 0), "wk": (KIND_HEAD, 0), "wv": (KIND_HEAD, 0), "wo": (KIND_HEAD, 1),
    "bq": (KIND_HEAD, 0), "bk": (KIND_HEAD, 0), "bv": (KIND_HEAD, 0),
    "w_up": (KIND_FFN, 0), "w_gate": (KIND_FFN, 0), "w_down": (KIND_FFN, 1), "b_up": (KIND_FFN, 0),
}


def _block_size(kind, d_head, granule):
    return d_head if kind == KIND_HEAD else granule


def element_index(row, q):
    """Element positions along the block axis covered by blueprint row `row` with block size q."""
    row = np.asarray(row, dtype=np.int64)
    return (row[:, None] * q + np.arange(q)[None, :]).reshape(-1)


def extract(full, plan, s, d_head, granule=1):
    """Subnet s of `full` = {"layers": [...], "globals": {...}} under `plan` (see sample.sample_plan)."""
    sub = {"layers": [], "globals": {k: v.copy() for k, v in full["globals"].items()}}
    for l, lw in enumerate(full["layers"]):
        out = {}
        for name, w in lw.items():
            if name in PARTITIONED:
                kind, axis = PARTITIONED[name]
                e = element_index(plan[l][kind]["idx"][s], _block_size(kind, d_head, granule))
                out[name] = np.take(w, e, axis=axis)
            else:
                out[name] = w.copy()
        sub["layers"].append(out)
    return sub


def aggregate(full, plan, subs, d_head, granule=1):
    """Return the new central model.  `subs` may be a subset of the S subnets given as {s: subnet};
    a list means subnets 0..len-1.  Written element by element from the formula: accumulate
    numerator and denominator, divide where the denominator is positive, else keep the old value."""
    if not isinstance(subs, dict):
        subs = dict(enumerate(subs))
    new = {"layers": [], "globals": {}}
    for name, w in full["globals"].items():
        new["globals"][name] = sum(sub["globals"][name] for sub in subs.values()) / len(subs)
    for l, lw in enumerate(full["layers"]):
        out = {}
        for name, w in lw.items():
            if name not in PARTITIONED:
                out[name] = sum(sub["layers"][l][name] for sub in subs.values()) / len(subs)
                continue
            kind, axis = PARTITIONED[name]
            q = _block_size(kind, d_head, granule)
            num = np.zeros_like(w)
            den = np.zeros(w.shape[axis])
            for s, sub in subs.items():
                e = element_index(plan[l][kind]["idx"][s], q)
                if axis == 0:
                    num[e] += sub["layers"][l][name]
                else:
                    num[:, e] += sub["layers"][l][name]
                den[e] += 1
            den_b = den[:, None] if (axis == 0 and w.ndim == 2) else den
            out[name] = np.where(den_b > 0, num / np.maximum(den_b, 1), w)
        new["layers"].append(out)
    return new
