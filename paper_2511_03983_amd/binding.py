"""ctypes binding with the same names as include/twist.h, plus small holder classes that keep the
torch tensors behind the raw pointers alive.  PyTorch is used for device memory and streams only."""
from __future__ import annotations

import ctypes as C
import os

import torch

__all__ = [
    "TwistError", "ModelDesc", "SampleDesc", "OptDesc", "lib", "Context", "Plan", "Subnet", "FullWeights",
    "LAYER_TENSORS", "GLOBAL_TENSORS", "F32", "BF16", "KIND_HEAD", "KIND_FFN", "STORE_PARAMS", "STORE_GRADS",
    "STORE_ADAMW", "OPT_SGD", "OPT_ADAMW", "SCALE_NONE", "SCALE_SQRT_RATIO", "desc_from_cfg",
]

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtwist.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or paper_2511_03983_amd/build.py) first; there is no fallback path")
lib = C.CDLL(_LIB_PATH)

F32, BF16 = 0, 1
ACT = {"gelu_tanh": 0, "relu": 1, "swiglu": 2}
NORM = {"ln": 0, "rms": 1}
KIND_HEAD, KIND_FFN = 0, 1
SCALE_NONE, SCALE_SQRT_RATIO = 0, 1
OPT_SGD, OPT_ADAMW = 0, 1
PARAM, GRAD, MASTER, ADAM_M, ADAM_V = 0, 1, 2, 3, 4
STORE_PARAMS, STORE_GRADS, STORE_ADAMW = 0, 1, 2
LAYER_TENSORS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "bq", "bk", "bv", "bo", "b_up", "b_down",
                 "norm1_w", "norm1_b", "norm2_w", "norm2_b")
GLOBAL_TENSORS = ("tok_embed", "pos_embed", "final_norm_w", "final_norm_b", "lm_head")
_STATUS = {1: "EINVAL", 2: "ECONSTRAINT", 3: "ESHAPE", 4: "ENOMEM", 5: "EHIP"}


class TwistError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"TWIST_{_STATUS.get(status, status)}: {msg}")
        self.status = status


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "d_head", "d_ff", "ffn_granule", "vocab",
                                         "max_seq", "act", "norm", "has_bias", "tied_head", "use_rope", "dtype", "out_unit_major")] + \
               [("norm_eps", C.c_float), ("rope_theta", C.c_float)]


class FullWeightsC(C.Structure):
    _fields_ = [("layer_tensors", C.POINTER(C.c_void_p)), ("global_tensors", C.c_void_p * len(GLOBAL_TENSORS))]


class SampleDesc(C.Structure):
    _fields_ = [("S", C.c_int32), ("heads_sub", C.c_int32), ("ffn_units_sub", C.c_int32),
                ("common_heads", C.POINTER(C.c_int32)), ("n_common_heads", C.c_int32),
                ("common_ffn", C.POINTER(C.c_int32)), ("n_common_ffn", C.c_int32),
                ("layer_shared", C.POINTER(C.c_uint8)), ("require_coverage", C.c_int32), ("scale_mode", C.c_int32),
                ("seed", C.c_uint64), ("round", C.c_uint64)]


class OptDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float)]


class RoundDesc(C.Structure):
    _fields_ = [("sample", SampleDesc), ("opt", OptDesc), ("local_steps", C.c_int32), ("B", C.c_int32), ("N", C.c_int32)]


_vp, _i32, _sz = C.c_void_p, C.c_int32, C.c_size_t
_PI32 = C.POINTER(C.c_int32)
_SIGS = {
    "twist_create": ([C.POINTER(ModelDesc), _vp, C.POINTER(_vp)], _i32),
    "twist_destroy": ([_vp], None),
    "twist_last_error": ([_vp], C.c_char_p),
    "twist_sample": ([_vp, C.POINTER(SampleDesc), C.POINTER(_vp)], _i32),
    "twist_plan_view": ([_vp, _i32, _i32, C.POINTER(_PI32), C.POINTER(_PI32), C.POINTER(_PI32), _PI32, _PI32, _i32], _i32),
    "twist_plan_read_device": ([_vp, _i32, _i32, _PI32, _PI32, _PI32], _i32),
    "twist_plan_destroy": ([_vp], None),
    "twist_subnet_bytes": ([_vp, _vp, _i32, C.POINTER(_sz)], _i32),
    "twist_extract": ([_vp, _vp, C.POINTER(FullWeightsC), _i32, _vp, _sz, _i32, C.POINTER(_vp)], _i32),
    "twist_extract_all": ([_vp, _vp, C.POINTER(FullWeightsC), C.POINTER(_vp), _sz, _i32, C.POINTER(_vp)], _i32),
    "twist_subnet_view": ([_vp, _i32, _i32, _i32, C.POINTER(_vp), C.POINTER(C.c_int64)], _i32),
    "twist_subnet_destroy": ([_vp], None),
    "twist_workspace_bytes": ([_vp, _vp, _i32, _i32, C.POINTER(_sz)], _i32),
    "twist_subnet_fwd_bwd": ([_vp, _vp, _vp, _vp, _i32, _i32, _vp, _sz, _vp], _i32),
    "twist_subnet_forward": ([_vp, _vp, _vp, _vp, _i32, _i32, _vp, _sz, _vp], _i32),
    "twist_subnet_fwd_bwd_masked": ([_vp, _vp, _vp, _i32, _vp, _vp, _i32, _i32, _vp, _sz, _vp], _i32),
    "twist_subnet_step": ([_vp, _vp, C.POINTER(OptDesc)], _i32),
    "twist_aggregate": ([_vp, _vp, C.POINTER(_vp), _i32, C.POINTER(FullWeightsC)], _i32),
    "twist_aggregate_image_bytes": ([_vp, C.POINTER(_sz)], _i32),
    "twist_aggregate_begin": ([_vp, _vp, _vp, _sz, C.POINTER(_vp)], _i32),
    "twist_aggregate_add": ([_vp, _vp], _i32),
    "twist_aggregate_finish": ([_vp, C.POINTER(FullWeightsC)], _i32),
    "twist_aggregate_destroy": ([_vp], None),
    "twist_round_bytes": ([_vp, C.POINTER(RoundDesc), C.POINTER(_sz), C.POINTER(_sz), C.POINTER(_sz)], _i32),
    "twist_round": ([_vp, C.POINTER(RoundDesc), C.POINTER(FullWeightsC), _vp, _vp, _vp, _sz, _vp, _sz, _vp, _sz, _vp], _i32),
    "twist_gemm_raw": ([_vp, _i32, _i32, _i32, _i32, _vp, C.c_int64, _vp, C.c_int64, _vp, C.c_int64, _i32, C.c_float], _i32),
    "twist_attention_raw": ([_vp, _vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp], _i32),
    "twist_norm_raw": ([_vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz], _i32),
    "twist_norm_raw_static": ([_vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp], _i32),
    "twist_rope_raw": ([_vp, _vp, _i32, _i32, _i32, C.c_float, _vp], _i32),
    "twist_act_raw": ([_vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _i32], _i32),
    "twist_ce_raw": ([_vp, _vp, C.c_int64, _vp, _i32, _vp, _vp], _i32),
    "twist_embed_raw": ([_vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp], _i32),
    "twist_set_kernel_choice": ([_vp, _i32, _i32, _i32], _i32),
    "twist_profile_gemm": ([_vp, _i32], _i32),
    "twist_set_overlap": ([_vp, _i32], _i32),
    "twist_profile_mfma_ceiling": ([_vp, _i32, _i32, _i32, _vp, _sz, C.POINTER(C.c_double)], _i32),
    "twist_profile_gemm_read": ([_vp, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)], _i32),
}
for _name, (_args, _res) in _SIGS.items():
    _f = getattr(lib, _name)          # AttributeError here = the library lacks a declared entry point
    _f.argtypes, _f.restype = _args, _res
EXPORTS = tuple(_SIGS)


def _ptr(t):
    """Device address of a tensor as a void pointer argument (None stays NULL)."""
    return None if t is None else _vp(t.data_ptr())


def _check(status, ctx=None):
    if status != 0:
        raise TwistError(status, (lib.twist_last_error(ctx) or b"").decode())


def desc_from_cfg(cfg) -> ModelDesc:
    """Build a ModelDesc from any object with the model-shape attributes (see include/twist.h)."""
    return ModelDesc(cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.d_head, cfg.d_ff, cfg.ffn_granule, cfg.vocab, cfg.max_seq,
                     ACT[cfg.act], NORM[cfg.norm], int(cfg.has_bias), int(cfg.tied_head), int(cfg.rope),
                     BF16 if cfg.dtype == "bf16" else F32, int(getattr(cfg, "out_unit_major", False)), cfg.norm_eps, cfg.rope_theta)


class Context:
    """twist_create / twist_destroy.  Work is enqueued on `stream` (default: torch's current stream)."""

    def __init__(self, desc: ModelDesc, stream: torch.cuda.Stream | None = None):
        self.desc = desc
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = _vp()
        _check(lib.twist_create(C.byref(desc), _vp(self.stream.cuda_stream), C.byref(h)))
        self.h = h
        self.torch_dtype = torch.bfloat16 if desc.dtype == BF16 else torch.float32

    def close(self):
        if getattr(self, "h", None):
            lib.twist_destroy(self.h)
            self.h = None

    __del__ = close

    # ---- the C entry points, by name -----------------------------------------------------------
    def twist_sample(self, S, heads_sub, ffn_units_sub, seed=0, rnd=0, common_heads=(), common_ffn=(), layer_shared=None,
                     require_coverage=True, scale_mode=SCALE_SQRT_RATIO) -> "Plan":
        ch = (C.c_int32 * len(common_heads))(*common_heads)
        cf = (C.c_int32 * len(common_ffn))(*common_ffn)
        ls = (C.c_uint8 * self.desc.n_layers)(*[int(bool(x)) for x in layer_shared]) if layer_shared is not None else None
        sd = SampleDesc(S, heads_sub, ffn_units_sub, ch, len(common_heads), cf, len(common_ffn), ls,
                        int(require_coverage), scale_mode, seed, rnd)
        h = _vp()
        _check(lib.twist_sample(self.h, C.byref(sd), C.byref(h)), self.h)
        return Plan(self, h, S)

    def twist_subnet_bytes(self, plan: "Plan", store=STORE_PARAMS) -> int:
        n = _sz()
        _check(lib.twist_subnet_bytes(self.h, plan.h, store, C.byref(n)), self.h)
        return n.value

    def twist_extract(self, plan: "Plan", full: "FullWeights", s: int, store=STORE_PARAMS, storage: torch.Tensor | None = None) -> "Subnet":
        if storage is None:
            storage = torch.empty(self.twist_subnet_bytes(plan, store), dtype=torch.uint8, device="cuda")
        h = _vp()
        _check(lib.twist_extract(self.h, plan.h, C.byref(full.c), s, _vp(storage.data_ptr()), storage.numel(), store, C.byref(h)), self.h)
        return Subnet(self, plan, h, storage, s)

    def twist_extract_all(self, plan: "Plan", full: "FullWeights", store=STORE_PARAMS, storages=None):
        """All S subnets of the plan in one pass over the central model; returns the list of Subnet holders."""
        if storages is None:
            nb = self.twist_subnet_bytes(plan, store)
            storages = [torch.empty(nb, dtype=torch.uint8, device="cuda") for _ in range(plan.S)]
        ptrs = (_vp * plan.S)(*[st.data_ptr() for st in storages])
        hs = (_vp * plan.S)()
        _check(lib.twist_extract_all(self.h, plan.h, C.byref(full.c), ptrs, min(st.numel() for st in storages), store, hs), self.h)
        return [Subnet(self, plan, _vp(hs[s]), storages[s], s) for s in range(plan.S)]

    def twist_workspace_bytes(self, sub: "Subnet", B: int, N: int) -> int:
        n = _sz()
        _check(lib.twist_workspace_bytes(self.h, sub.h, B, N, C.byref(n)), self.h)
        return n.value

    def twist_subnet_fwd_bwd(self, sub: "Subnet", inputs: torch.Tensor, targets: torch.Tensor, workspace: torch.Tensor,
                             loss: torch.Tensor) -> None:
        B, N = inputs.shape[0], inputs.shape[1]
        _check(lib.twist_subnet_fwd_bwd(self.h, sub.h, _vp(inputs.data_ptr()), _vp(targets.data_ptr()), B, N,
                                        _vp(workspace.data_ptr()), workspace.numel(), _vp(loss.data_ptr())), self.h)

    def twist_subnet_fwd_bwd_masked(self, full_sub: "Subnet", plan: "Plan", s: int, inputs: torch.Tensor, targets: torch.Tensor,
                                    workspace: torch.Tensor, loss: torch.Tensor) -> None:
        B, N = inputs.shape[0], inputs.shape[1]
        _check(lib.twist_subnet_fwd_bwd_masked(self.h, full_sub.h, plan.h, s, _vp(inputs.data_ptr()), _vp(targets.data_ptr()), B, N,
                                               _vp(workspace.data_ptr()), workspace.numel(), _vp(loss.data_ptr())), self.h)

    def twist_subnet_forward(self, sub: "Subnet", inputs: torch.Tensor, targets: torch.Tensor, workspace: torch.Tensor,
                             loss: torch.Tensor) -> None:
        B, N = inputs.shape[0], inputs.shape[1]
        _check(lib.twist_subnet_forward(self.h, sub.h, _vp(inputs.data_ptr()), _vp(targets.data_ptr()), B, N,
                                        _vp(workspace.data_ptr()), workspace.numel(), _vp(loss.data_ptr())), self.h)

    def twist_subnet_step(self, sub: "Subnet", kind=OPT_SGD, lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0) -> None:
        od = OptDesc(kind, lr, beta1, beta2, eps, weight_decay)
        _check(lib.twist_subnet_step(self.h, sub.h, C.byref(od)), self.h)

    def twist_aggregate(self, plan: "Plan", subs, full: "FullWeights") -> None:
        arr = (_vp * len(subs))(*[s.h for s in subs])
        _check(lib.twist_aggregate(self.h, plan.h, arr, len(subs), C.byref(full.c)), self.h)

    def twist_aggregate_image_bytes(self) -> int:
        n = _sz()
        _check(lib.twist_aggregate_image_bytes(self.h, C.byref(n)), self.h)
        return n.value

    def twist_aggregate_begin(self, plan: "Plan", image: torch.Tensor | None = None) -> "Accum":
        if image is None:
            image = torch.empty(self.twist_aggregate_image_bytes(), dtype=torch.uint8, device="cuda")
        h = _vp()
        _check(lib.twist_aggregate_begin(self.h, plan.h, _vp(image.data_ptr()), image.numel(), C.byref(h)), self.h)
        return Accum(self, plan, h, image)

    def _round_desc(self, S, heads_sub, ffn_units_sub, B, N, local_steps, seed, rnd, opt, layer_shared, scale_mode):
        keep = []
        ls = None
        if layer_shared is not None:
            ls = (C.c_uint8 * self.desc.n_layers)(*[int(bool(x)) for x in layer_shared])
            keep.append(ls)
        sd = SampleDesc(S, heads_sub, ffn_units_sub, None, 0, None, 0, ls, 1, scale_mode, seed, rnd)
        od = OptDesc(opt.get("kind", OPT_SGD), opt.get("lr", 1e-2), opt.get("beta1", 0.9), opt.get("beta2", 0.999), opt.get("eps", 1e-8),
                     opt.get("weight_decay", 0.0))
        return RoundDesc(sd, od, local_steps, B, N), keep

    def twist_round_bytes(self, S, heads_sub, ffn_units_sub, B, N, local_steps=1, seed=0, rnd=0, opt=None, layer_shared=None,
                          scale_mode=SCALE_SQRT_RATIO):
        """(subnet_bytes, workspace_bytes, image_bytes) of twist_round with these arguments."""
        rd, _keep = self._round_desc(S, heads_sub, ffn_units_sub, B, N, local_steps, seed, rnd, opt or {}, layer_shared, scale_mode)
        a, b, c = _sz(), _sz(), _sz()
        _check(lib.twist_round_bytes(self.h, C.byref(rd), C.byref(a), C.byref(b), C.byref(c)), self.h)
        return a.value, b.value, c.value

    def twist_round(self, full: "FullWeights", inputs: torch.Tensor, targets: torch.Tensor, S, heads_sub, ffn_units_sub, subnet_storage,
                    workspace, image, loss, seed=0, rnd=0, opt=None, layer_shared=None, scale_mode=SCALE_SQRT_RATIO) -> None:
        """inputs/targets [S, local_steps, B, N(, d_model)]; loss fp32 [S, local_steps] (device)."""
        local_steps, B, N = inputs.shape[1], inputs.shape[2], inputs.shape[3]
        rd, _keep = self._round_desc(S, heads_sub, ffn_units_sub, B, N, local_steps, seed, rnd, opt or {}, layer_shared, scale_mode)
        _check(lib.twist_round(self.h, C.byref(rd), C.byref(full.c), _vp(inputs.data_ptr()), _vp(targets.data_ptr()),
                               _vp(subnet_storage.data_ptr()), subnet_storage.numel(), _vp(workspace.data_ptr()), workspace.numel(),
                               _vp(image.data_ptr()), image.numel(), _vp(loss.data_ptr())), self.h)


    def twist_gemm_raw(self, layout: int, M: int, N: int, K: int, A: torch.Tensor, B: torch.Tensor, out: torch.Tensor, alpha: float = 1.0) -> None:
        """out[M,N] = alpha * op(A) op(B); layouts as in include/twist.h; row strides taken from the tensors."""
        _check(lib.twist_gemm_raw(self.h, layout, M, N, K, _vp(A.data_ptr()), A.stride(0), _vp(B.data_ptr()), B.stride(0),
                                  _vp(out.data_ptr()), out.stride(0), int(out.dtype == torch.float32 and self.torch_dtype != torch.float32
                                                                          or out.dtype == torch.float32), alpha), self.h)

    def twist_attention_raw(self, qkv: torch.Tensor, dout, B: int, N: int, Hs: int, keep: torch.Tensor | None = None, rope_backward: bool = False):
        """Causal attention alone: returns (o, lse, dqkv or None) for qkv [B*N, 3*Hs*d_head] and dout [B*N, Hs*d_head] or None;
        keep: int32 [Hs] head mask (entries < 0 are masked) or None; rope_backward: the q and k gradients are also turned
        back through the rotary embedding."""
        T, HD = B * N, qkv.shape[1] // 3
        o = torch.empty((T, HD), dtype=qkv.dtype, device=qkv.device)
        o32 = torch.empty((T, HD), dtype=torch.float32, device=qkv.device)
        lse = torch.empty((B, Hs, N), dtype=torch.float32, device=qkv.device)
        delta = torch.empty_like(lse)
        dqkv = torch.empty_like(qkv) if dout is not None else None
        _check(lib.twist_attention_raw(self.h, _vp(qkv.data_ptr()), _vp(dout.data_ptr()) if dout is not None else None, B, N, Hs,
                                       _vp(o.data_ptr()), _vp(o32.data_ptr()), _vp(lse.data_ptr()), _vp(delta.data_ptr()),
                                       _vp(dqkv.data_ptr()) if dqkv is not None else None, _ptr(keep),
                                       _ptr(torch.empty(N * self.desc.d_head, dtype=torch.float32, device=qkv.device)) if rope_backward else None), self.h)
        return o, lse, dqkv

    def twist_norm_raw(self, x: torch.Tensor, w: torch.Tensor, b, dy=None):
        """y = f_ln(x) for x fp32 [T, d_model]; with dy also (dx fp32, dxb, dw, db or None).  Returns (y, stats, backward tuple or None)."""
        T, D = x.shape
        y = torch.empty((T, D), dtype=self.torch_dtype, device=x.device)
        stats = torch.empty((T, 2), dtype=torch.float32, device=x.device)
        if dy is None:
            _check(lib.twist_norm_raw(self.h, _ptr(x), _ptr(w), _ptr(b), T, _ptr(y), _ptr(stats), None, None, None, None, None, None, 0), self.h)
            return y, stats, None
        dx = torch.empty_like(x)
        dxb = torch.empty_like(y)
        dw = torch.empty(D, dtype=torch.float32, device=x.device)
        db = torch.empty(D, dtype=torch.float32, device=x.device) if b is not None else None
        scratch = torch.empty(((T + 15) // 16) * 2 * D, dtype=torch.float32, device=x.device)
        _check(lib.twist_norm_raw(self.h, _ptr(x), _ptr(w), _ptr(b), T, _ptr(y), _ptr(stats), _ptr(dy), _ptr(dx), _ptr(dxb), _ptr(dw), _ptr(db),
                                  _ptr(scratch), scratch.numel()), self.h)
        return y, stats, (dx, dxb, dw, db)

    def twist_norm_raw_static(self, x, w, b, dy, y, stats, dx, dxb, dw, db) -> None:
        """twist_norm_raw on caller-provided outputs with the library's built-in scratch: the call allocates nothing."""
        _check(lib.twist_norm_raw_static(self.h, _ptr(x), _ptr(w), _ptr(b), x.shape[0], _ptr(y), _ptr(stats), _ptr(dy), _ptr(dx), _ptr(dxb),
                                         _ptr(dw), _ptr(db)), self.h)

    def twist_rope_raw(self, qkv: torch.Tensor, B: int, N: int, Hs: int, sign: float = 1.0) -> None:
        """Rotary positions applied in place to the q and k heads of qkv [B*N, 3*Hs*d_head]."""
        tab = torch.empty(N * self.desc.d_head, dtype=torch.float32, device=qkv.device)
        _check(lib.twist_rope_raw(self.h, _ptr(qkv), B, N, Hs, sign, _ptr(tab)), self.h)

    def twist_act_raw(self, gu: torch.Tensor, F: int, da=None, keep=None, unit: int = 1):
        """(a, dgu or None): the FFN activation on gu [T, F] (or [T, 2F] gate | up) and its backward for da [T, F]."""
        T = gu.shape[0]
        a = torch.empty((T, F), dtype=gu.dtype, device=gu.device)
        dgu = torch.empty_like(gu) if da is not None else None
        _check(lib.twist_act_raw(self.h, _ptr(gu), T, F, _ptr(a), _ptr(da), _ptr(dgu), _ptr(keep), unit), self.h)
        return a, dgu

    def twist_ce_raw(self, logits: torch.Tensor, targets: torch.Tensor):
        """Mean cross-entropy of logits [T, ld] (overwritten by its gradient); returns (loss tensor, rowloss)."""
        T = logits.shape[0]
        rowloss = torch.empty(max(T, 1024), dtype=torch.float32, device=logits.device)
        loss = torch.zeros(1, dtype=torch.float32, device=logits.device)
        _check(lib.twist_ce_raw(self.h, _ptr(logits), logits.stride(0), _ptr(targets), T, _ptr(rowloss), _ptr(loss)), self.h)
        return loss, rowloss[:T]

    def twist_embed_raw(self, tok: torch.Tensor, tok_embed: torch.Tensor, pos_embed=None, dx=None):
        """x fp32 [B*N, d_model] = embedding rows (+ positions); with dx also (d_tok, d_pos or None)."""
        B, N = tok.shape
        D = tok_embed.shape[1]
        x = torch.empty((B * N, D), dtype=torch.float32, device=tok.device)
        d_tok = torch.zeros(tok_embed.shape, dtype=torch.float32, device=tok.device) if dx is not None else None
        d_pos = torch.empty((N, D), dtype=torch.float32, device=tok.device) if (dx is not None and pos_embed is not None) else None
        _check(lib.twist_embed_raw(self.h, _ptr(tok), B, N, _ptr(tok_embed), _ptr(pos_embed), _ptr(x), _ptr(dx), _ptr(d_tok), _ptr(d_pos)), self.h)
        return x, d_tok, d_pos

    def twist_set_kernel_choice(self, gemm_tile: int = 0, plain_only: bool = False, staged_attention: bool = False) -> None:
        _check(lib.twist_set_kernel_choice(self.h, gemm_tile, int(plain_only), int(staged_attention)), self.h)

    def twist_set_overlap(self, enable: bool) -> None:
        _check(lib.twist_set_overlap(self.h, int(enable)), self.h)

    def twist_profile_mfma_ceiling(self, waves_per_simd: int = 2, iters: int = 20000, random_operands: bool = True) -> float:
        """TFLOP/s of the bf16 matrix instruction alone on the whole chip (no loads)."""
        sink = torch.empty(1024 * 8 * 256, dtype=torch.float32, device="cuda")
        tf = C.c_double()
        _check(lib.twist_profile_mfma_ceiling(self.h, waves_per_simd, iters, int(random_operands), _ptr(sink), sink.numel(), C.byref(tf)), self.h)
        return tf.value

    def twist_profile_gemm(self, enable: bool) -> None:
        _check(lib.twist_profile_gemm(self.h, int(enable)), self.h)

    def twist_profile_gemm_read(self):
        """(launches, milliseconds, algorithmic flops) of the projection kernels since enabling."""
        n, ms, fl = C.c_int64(), C.c_double(), C.c_double()
        _check(lib.twist_profile_gemm_read(self.h, C.byref(n), C.byref(ms), C.byref(fl)), self.h)
        return n.value, ms.value, fl.value


class Plan:
    def __init__(self, ctx: Context, h, S):
        self.ctx, self.h, self.S = ctx, h, S

    def twist_plan_view(self, layer: int, kind: int):
        """Host copies of (idx [S, n_sub], inv [S, n_full], count [n_full]) as int32 torch tensors."""
        idx, inv, cnt = _PI32(), _PI32(), _PI32()
        ns, nf = C.c_int32(), C.c_int32()
        _check(lib.twist_plan_view(self.h, layer, kind, C.byref(idx), C.byref(inv), C.byref(cnt), C.byref(ns), C.byref(nf), 0), self.ctx.h)
        S, ns, nf = self.S, ns.value, nf.value
        as_t = lambda p, n: torch.tensor(p[:n], dtype=torch.int32)
        return as_t(idx, S * ns).view(S, ns), as_t(inv, S * nf).view(S, nf), as_t(cnt, nf)

    def twist_plan_read_device(self, layer: int, kind: int):
        """(idx [S, n_sub], inv [S, n_full], count [n_full]) as int32 torch tensors, copied back from the DEVICE tables."""
        _, _, _, ns, nf = self.device_tables(layer, kind)
        idx, inv, cnt = (C.c_int32 * (self.S * ns))(), (C.c_int32 * (self.S * nf))(), (C.c_int32 * nf)()
        _check(lib.twist_plan_read_device(self.h, layer, kind, idx, inv, cnt), self.ctx.h)
        as_t = lambda a: torch.tensor(list(a), dtype=torch.int32)
        return as_t(idx).view(self.S, ns), as_t(inv).view(self.S, nf), as_t(cnt)

    def device_tables(self, layer: int, kind: int):
        """Raw device addresses of (idx, inv, count) and (n_sub, n_full)."""
        idx, inv, cnt = _PI32(), _PI32(), _PI32()
        ns, nf = C.c_int32(), C.c_int32()
        _check(lib.twist_plan_view(self.h, layer, kind, C.byref(idx), C.byref(inv), C.byref(cnt), C.byref(ns), C.byref(nf), 1), self.ctx.h)
        addr = lambda p: C.cast(p, C.c_void_p).value
        return addr(idx), addr(inv), addr(cnt), ns.value, nf.value

    def close(self):
        if getattr(self, "h", None):
            lib.twist_plan_destroy(self.h)
            self.h = None

    __del__ = close


class Accum:
    """twist_aggregate_begin / add / finish / destroy: the aggregation one subnet at a time."""

    def __init__(self, ctx: Context, plan: "Plan", h, image: torch.Tensor):
        self.ctx, self.plan, self.h, self.image = ctx, plan, h, image

    def twist_aggregate_add(self, sub: "Subnet") -> None:
        _check(lib.twist_aggregate_add(self.h, sub.h), self.ctx.h)

    def twist_aggregate_finish(self, full: "FullWeights") -> None:
        _check(lib.twist_aggregate_finish(self.h, C.byref(full.c)), self.ctx.h)

    def close(self):
        if getattr(self, "h", None):
            lib.twist_aggregate_destroy(self.h)
            self.h = None

    __del__ = close


class Subnet:
    def __init__(self, ctx: Context, plan: Plan, h, storage: torch.Tensor, s: int):
        self.ctx, self.plan, self.h, self.storage, self.s = ctx, plan, h, storage, s

    def twist_subnet_view(self, layer: int, tensor: str | int, what=PARAM) -> torch.Tensor:
        """A torch view (no copy) of one subnet tensor inside the caller-owned storage."""
        names = GLOBAL_TENSORS if layer < 0 else LAYER_TENSORS
        t = names.index(tensor) if isinstance(tensor, str) else tensor
        dev, shape = _vp(), (C.c_int64 * 2)()
        _check(lib.twist_subnet_view(self.h, layer, t, what, C.byref(dev), shape), self.ctx.h)
        dt = self.ctx.torch_dtype if what == PARAM else torch.float32      # gradient, master weights and moments are fp32
        n = shape[0] * shape[1]
        off = dev.value - self.storage.data_ptr()
        v = self.storage[off: off + n * dt.itemsize].view(dt)
        is_matrix = names[t] in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "tok_embed", "pos_embed", "lm_head")
        return v.view(shape[0], shape[1]) if (shape[1] > 1 or is_matrix) else v      # a one-column matrix stays a matrix

    def has(self, layer: int, tensor: str) -> bool:
        try:
            self.twist_subnet_view(layer, tensor)
            return True
        except TwistError:
            return False

    def close(self):
        if getattr(self, "h", None):
            lib.twist_subnet_destroy(self.h)
            self.h = None

    __del__ = close


class FullWeights:
    """Pointer table over caller-owned torch tensors: layers = [ {name: tensor} ], globals_ = {name: tensor}."""

    def __init__(self, layers, globals_=None):
        self.layers, self.globals = layers, dict(globals_ or {})
        n = len(layers) * len(LAYER_TENSORS)
        self._arr = (C.c_void_p * n)()
        for l, lw in enumerate(layers):
            for t, name in enumerate(LAYER_TENSORS):
                w = lw.get(name)
                if w is not None:
                    assert w.is_cuda and w.is_contiguous()
                    self._arr[l * len(LAYER_TENSORS) + t] = w.data_ptr()
        g = (C.c_void_p * len(GLOBAL_TENSORS))()
        for t, name in enumerate(GLOBAL_TENSORS):
            w = self.globals.get(name)
            if w is not None:
                assert w.is_cuda and w.is_contiguous()
                g[t] = w.data_ptr()
        self.c = FullWeightsC(C.cast(self._arr, C.POINTER(C.c_void_p)), g)
