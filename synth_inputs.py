"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only *generates data* (weights, activations, token ids, perturbations).
It holds none of the method's arithmetic: no sampling of subnets, no gathers, no
model math.  Every array is a pure function of (seed, name), drawn from numpy's
counter-based Philox generator, so the CPU checker and the GPU path can be fed
identical inputs without either seeing the other's code.

Shapes follow the GPT-style workloads of the paper's experiments (Section 5,
"Setup": 12-layer / 12-head / 768-wide GPT-2, 1024-token sequences) and their
Llama-shaped scale-ups; layouts are [out_features, in_features] row-major (the mathematical
shapes; `stored_shapes` gives the memory layout a configuration asks the library to use).
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field, replace

import numpy as np

# tensor names, per layer
LAYER_MATS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")
LAYER_VECS = ("bq", "bk", "bv", "bo", "b_up", "b_down",
              "norm1_w", "norm1_b", "norm2_w", "norm2_b")
GLOBALS = ("tok_embed", "pos_embed", "final_norm_w", "final_norm_b", "lm_head")


@dataclass(frozen=True)
class ModelCfg:
    arch: str = "gpt"           # "gpt" | "llama"
    n_layers: int = 1
    d_model: int = 128
    n_heads: int = 4
    d_head: int = 32
    d_ff: int = 512
    ffn_granule: int = 1        # neurons per FFN block (d_ff / R)
    vocab: int = 0              # 0 = block-stack mode: activations in, MSE loss
    max_seq: int = 64
    act: str = "gelu_tanh"      # "gelu_tanh" | "relu" | "swiglu"
    norm: str = "ln"            # "ln" | "rms"
    has_bias: bool = True
    tied_head: bool = True
    rope: bool = False
    dtype: str = "f32"          # "f32" | "bf16"
    norm_eps: float = 1e-5
    rope_theta: float = 10000.0
    out_unit_major: bool = False  # the library stores wo and w_down transposed ([in, out]); the maths is unchanged

    @property
    def n_ffn_units(self) -> int:
        return self.d_ff // self.ffn_granule


# The five workload shapes (full size).  Tests shrink them with `replace`.
CFG1 = ModelCfg()
CFG2 = ModelCfg(arch="gpt", n_layers=12, d_model=768, n_heads=12, d_head=64, d_ff=3072,
                vocab=50257, max_seq=1024, dtype="bf16")
CFG3 = ModelCfg(arch="llama", n_layers=22, d_model=2048, n_heads=16, d_head=128, d_ff=5632,
                vocab=32000, max_seq=2048, act="swiglu", norm="rms", has_bias=False,
                tied_head=False, rope=True, dtype="bf16")
CFG4 = ModelCfg(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_head=128, d_ff=11008,
                vocab=0, max_seq=4096, act="swiglu", norm="rms", has_bias=False,
                tied_head=False, rope=True, dtype="bf16")
CFG5 = replace(CFG4, vocab=32000)


def _rng(seed: int, name: str) -> np.random.Generator:
    key = (int(seed) & 0xFFFFFFFF) << 32 | zlib.crc32(name.encode())
    return np.random.Generator(np.random.Philox(key=key))


def normal(seed: int, name: str, shape, std: float = 1.0) -> np.ndarray:
    """fp64 N(0, std^2) array, a pure function of (seed, name, shape)."""
    return _rng(seed, name).standard_normal(shape) * std


def to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Round fp64 values to the nearest bf16-representable value (ties to even), kept as fp64.

    Used so that bf16 workloads hand both sides *exactly* the same numbers.
    """
    f = np.asarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def layer_shapes(cfg: ModelCfg) -> dict:
    d, hd, f = cfg.d_model, cfg.n_heads * cfg.d_head, cfg.d_ff
    s = {"wq": (hd, d), "wk": (hd, d), "wv": (hd, d), "wo": (d, hd),
         "w_up": (f, d), "w_down": (d, f), "norm1_w": (d,), "norm2_w": (d,)}
    if cfg.act == "swiglu":
        s["w_gate"] = (f, d)
    if cfg.norm == "ln":
        s["norm1_b"] = (d,)
        s["norm2_b"] = (d,)
    if cfg.has_bias:
        s.update(bq=(hd,), bk=(hd,), bv=(hd,), bo=(d,), b_up=(f,), b_down=(d,))
    return s


STORED_TRANSPOSED = ("wo", "w_down")


def stored_shapes(cfg: ModelCfg) -> dict:
    """Shapes as the library stores them: with `out_unit_major` the two output projections are kept transposed."""
    s = layer_shapes(cfg)
    if cfg.out_unit_major:
        for k in STORED_TRANSPOSED:
            s[k] = s[k][::-1]
    return s


def global_shapes(cfg: ModelCfg) -> dict:
    if cfg.vocab == 0:
        return {}
    d = cfg.d_model
    s = {"tok_embed": (cfg.vocab, d), "final_norm_w": (d,)}
    if not cfg.rope:
        s["pos_embed"] = (cfg.max_seq, d)
    if cfg.norm == "ln":
        s["final_norm_b"] = (d,)
    if not cfg.tied_head:
        s["lm_head"] = (cfg.vocab, d)
    return s


def make_weights(cfg: ModelCfg, seed: int = 0, std: float = 0.02, generic: bool = False) -> dict:
    """Full-model weights: {"layers": [ {name: array} ], "globals": {name: array}} in fp64.

    Matrices ~ N(0, std); norm gains 1 and biases 0 as in a fresh GPT-style model, unless
    `generic` is set, in which case gains and biases are random too (so that tests can tell
    them apart).  For bf16 configs the values are snapped to the bf16 grid.
    """
    snap = to_bf16_grid if cfg.dtype == "bf16" else (lambda a: np.asarray(a, np.float32).astype(np.float64))
    layers = []
    for l in range(cfg.n_layers):
        lw = {}
        for name, shp in layer_shapes(cfg).items():
            if len(shp) == 2:
                a = normal(seed, f"L{l}.{name}", shp, std)
            elif name.endswith("_w") and name.startswith("norm"):
                a = 1.0 + (normal(seed, f"L{l}.{name}", shp, 0.1) if generic else 0.0) * np.ones(shp)
            else:
                a = normal(seed, f"L{l}.{name}", shp, 0.1) if generic else np.zeros(shp)
            lw[name] = snap(a)
        layers.append(lw)
    g = {}
    for name, shp in global_shapes(cfg).items():
        if len(shp) == 2:
            a = normal(seed, f"G.{name}", shp, std)
        elif name.endswith("_w"):
            a = 1.0 + (normal(seed, f"G.{name}", shp, 0.1) if generic else 0.0) * np.ones(shp)
        else:
            a = normal(seed, f"G.{name}", shp, 0.1) if generic else np.zeros(shp)
        g[name] = snap(a)
    return {"layers": layers, "globals": g}


def activations(cfg: ModelCfg, B: int, N: int, seed: int, name: str = "x") -> np.ndarray:
    """N(0,1) activations or regression targets [B, N, d_model] for block-stack mode."""
    a = normal(seed, f"act.{name}", (B, N, cfg.d_model), 1.0)
    return to_bf16_grid(a) if cfg.dtype == "bf16" else np.asarray(a, np.float32).astype(np.float64)


def tokens_uniform(vocab: int, B: int, N: int, seed: int, name: str = "tok"):
    """Uniform token ids [B, N+1]; callers slice inputs [:, :-1] and next-token targets [:, 1:]."""
    return _rng(seed, f"tok.{name}").integers(0, vocab, size=(B, N + 1), dtype=np.int64).astype(np.int32)


def tokens_zipf(vocab: int, B: int, N: int, seed: int, name: str = "tok", a: float = 1.1):
    """Token ids [B, N+1] with P(rank k) ~ k^-a, k = 1..vocab, id = k-1 (inverse-CDF sampling)."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-a)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = _rng(seed, f"zipf.{name}").random((B, N + 1))
    return np.minimum(np.searchsorted(cdf, u), vocab - 1).astype(np.int32)


def perturbation(seed: int, name: str, shape, std: float = 1e-3) -> np.ndarray:
    """N(0, std) noise standing in for a subnet's local training update."""
    return normal(seed, f"perturb.{name}", shape, std)
