"""Literal end-to-end tolerances of the bf16 path, from a count of rounding points (no reference run is involved).

The stated tolerance of a bf16-in / fp32-accumulate kernel is a relative Frobenius error of 5e-3, and every kernel is
held to it on its own (tests/test_gpu_kernels.py, test_gpu_gemm.py, test_gpu_fullsize.py).  End to end a gradient is
the product of two operands that each went through a chain of kernels, every one of which stored its result in bf16:

  eps      = 2^-9 / sqrt(3) = 1.13e-3   rms relative error of one round-to-nearest-even to 8 significant bits
  N(G)     = number of bf16 rounding points in the causal past of gradient tensor G (both operands of the
             contraction that forms it; the loss gradient depends on every forward rounding of the model)
  err(G)  ~= eps * sqrt(N(G))           independent roundings add in quadrature; contractions of random-sign terms,
                                         norms and residual adds pass a relative perturbation on with gain ~1
  bound(G) = min(1e-2, K * A(G) * eps * sqrt(N(G)))
  K        = 1.5   head room for the places where the gain is above 1 (the cancellations in the norm backward and in
                   softmax - onehot)
  A(G)     = 1.4 for the query / key weight and bias gradients, else 1: dS = P (dP - delta) cancels most of dP, so a
             relative error of dP or delta grows by |dP| / |dP - delta|

Rounding points of the library's bf16 pass, per layer (the checker's rounding hook offers the same list, pinned by
tests/test_oracle_model.py):
  forward   attention: normed input, q|k|v (+1 when rotary positions re-round q and k), probabilities inside the
            attention kernel, attention output = 4 (+1);  FFN: normed input, pre-activations, activation = 3
  backward  FFN branch: residual gradient handed in, gradient of the activation, of the pre-activations, of the normed
            input = 4;  attention branch: residual gradient, gradient of the attention output, dS inside the kernel,
            gradient of q|k|v, of the normed input = 5
  head      forward: final normed input, logits = 2;  backward: dlogits, gradient of the final normed input = 2
            (block-stack mode with the squared-error loss: none)
"""
import math

EPS = 2.0 ** -9 / math.sqrt(3.0)
K = 1.5
CAP = 1e-2
QK_GAIN = 1.4

# rounding points between the top of layer l's backward pass and the contraction that forms each gradient
_WITHIN = {
    "w_down": 1, "b_down": 1,
    "w_up": 3, "w_gate": 3, "b_up": 3,
    "norm2_w": 4, "norm2_b": 4,
    "wo": 5, "bo": 5,
    "wq": 8, "wk": 8, "wv": 8, "bq": 8, "bk": 8, "bv": 8,
    "norm1_w": 9, "norm1_b": 9,
}
_PER_LAYER_BWD = 9


def rounding_points(cfg, layer, name):
    """N(G) for layer tensor `name` of layer `layer` (0-based), or for a model-level tensor when layer < 0."""
    L = cfg.n_layers
    fwd_all = L * (7 + int(cfg.rope)) + (2 if cfg.vocab else 0)
    head_bwd = 2 if cfg.vocab else 0
    if layer < 0:
        if name == "lm_head":
            return fwd_all + 1
        if name in ("final_norm_w", "final_norm_b"):
            return fwd_all + 2
        return fwd_all + head_bwd + _PER_LAYER_BWD * L      # embeddings: the gradient that leaves layer 0
    return fwd_all + head_bwd + _PER_LAYER_BWD * (L - 1 - layer) + _WITHIN[name]


def bound(cfg, layer, name):
    gain = QK_GAIN if name in ("wq", "wk", "bq", "bk") else 1.0
    return min(CAP, K * gain * EPS * math.sqrt(rounding_points(cfg, layer, name)))


def bound_between_two_bf16_runs(cfg, layer, name):
    """Two results that are each within bound() of exact arithmetic, with independent rounding errors."""
    return math.sqrt(2.0) * bound(cfg, layer, name)
