"""Shared plumbing for the GPU parity tests: move seeded inputs to the device, read results back."""
import numpy as np
import torch

import synth_inputs as si


def torch_dtype(cfg):
    return torch.bfloat16 if cfg.dtype == "bf16" else torch.float32


def _stored(cfg, k, a):
    """[out, in] array <-> the layout the library keeps it in (a transpose for the output projections of a
    unit-major configuration; its own inverse)."""
    return a.T if cfg.out_unit_major and k in si.STORED_TRANSPOSED else a


def to_device(full_np, cfg):
    """numpy fp64 model (values already on the dtype's grid) -> dict of CUDA tensors in the stored layout."""
    dt = torch_dtype(cfg)
    conv = lambda a: torch.tensor(np.ascontiguousarray(a), dtype=torch.float64).to(dt).cuda().contiguous()
    return {"layers": [{k: conv(_stored(cfg, k, v)) for k, v in lw.items()} for lw in full_np["layers"]],
            "globals": {k: conv(v) for k, v in full_np["globals"].items()}}


def to_numpy(t):
    return t.detach().to(torch.float64).cpu().numpy()


def model_to_numpy(full_t, cfg=None):
    """Device model back to [out, in] numpy arrays."""
    back = (lambda k, a: _stored(cfg, k, a)) if cfg is not None else (lambda k, a: a)
    return {"layers": [{k: back(k, to_numpy(v)) for k, v in lw.items()} for lw in full_t["layers"]],
            "globals": {k: to_numpy(v) for k, v in full_t["globals"].items()}}


def subnet_to_numpy(sub, cfg, what=0):
    """Read every tensor of a library subnet back through twist_subnet_view, in the oracle's nesting and [out, in]."""
    out = {"layers": [], "globals": {}}
    for l in range(cfg.n_layers):
        out["layers"].append({k: _stored(cfg, k, to_numpy(sub.twist_subnet_view(l, k, what))) for k in si.layer_shapes(cfg)})
    for k in si.global_shapes(cfg):
        out["globals"][k] = to_numpy(sub.twist_subnet_view(-1, k, what))
    return out


def rel_fro(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def bf16_ulp_distance(a, b):
    """Distance in bf16 ulps between two arrays of bf16-representable fp64 values."""
    def key(x):
        u = np.asarray(x, np.float32).view(np.uint32).astype(np.int64) >> 16
        return np.where(u & 0x8000, 0x8000 - u, u)      # monotone integer order
    return np.abs(key(a) - key(b))
