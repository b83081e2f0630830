"""twist_norm_raw_static (the variant of twist_norm_raw for callers that cannot allocate: scratch in a built-in device
array) against twist_norm_raw, through the C ABI: same kernels, so every output must agree bit for bit; two calls in a
row, the second on a smaller input, and the size limit."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


def _case(lib, kind, D, T, seed):
    cfg = si.ModelCfg(d_model=D, n_heads=1, d_head=8, d_ff=8, norm=kind, dtype="bf16")
    ctx = lib.Context(lib.desc_from_cfg(cfg))
    g = torch.Generator(device="cuda").manual_seed(seed)
    x = torch.randn((T, D), generator=g, device="cuda") * 1.5 + 0.3
    w = (1.0 + 0.2 * torch.randn(D, generator=g, device="cuda")).to(torch.bfloat16)
    b = (0.2 * torch.randn(D, generator=g, device="cuda")).to(torch.bfloat16) if kind == "ln" else None
    dy = torch.randn((T, D), generator=g, device="cuda").to(torch.bfloat16)
    return ctx, x, w, b, dy


def _both(lib, kind, D, T, seed):
    ctx, x, w, b, dy = _case(lib, kind, D, T, seed)
    y0, stats0, (dx0, dxb0, dw0, db0) = ctx.twist_norm_raw(x, w, b, dy)
    nan = float("nan")
    y, dxb = torch.full_like(y0, nan), torch.full_like(dxb0, nan)
    stats, dx, dw = torch.full_like(stats0, nan), torch.full_like(dx0, nan), torch.full_like(dw0, nan)
    db = torch.full_like(db0, nan) if db0 is not None else None
    ctx.twist_norm_raw_static(x, w, b, dy, y, stats, dx, dxb, dw, db)
    torch.cuda.synchronize()
    for name, a, c in (("y", y, y0), ("stats", stats, stats0), ("dx", dx, dx0), ("dxb", dxb, dxb0), ("dw", dw, dw0)) + ((("db", db, db0),) if db is not None else ()):
        assert torch.equal(a.view(torch.uint8), c.view(torch.uint8)), (kind, D, T, name)
    assert torch.isfinite(dw).all() and float(dw.abs().max()) > 0


def test_static_scratch_variant_equals_the_caller_scratch_entry_point(lib):
    _both(lib, "rms", 2048, 1000, 1)      # 63 chunks of 16 rows
    _both(lib, "ln", 256, 37, 2)          # right after it, a smaller input: stale partial sums of the first call must not leak in
    _both(lib, "ln", 200, 50, 3)          # the general kernels
    _both(lib, "rms", 4096, 4096, 4)      # exactly the limit: 256 chunks * 2 * 4096 floats


def test_static_scratch_variant_rejects_sizes_beyond_its_array(lib):
    ctx, x, w, b, dy = _case(lib, "rms", 4096, 4112, 5)      # 257 chunks: one more than the array holds
    out = [torch.empty_like(t) for t in (dy, x[:, :2].contiguous(), x, dy, x[0], x[0])]
    with pytest.raises(lib.TwistError) as e:
        ctx.twist_norm_raw_static(x, w, None, dy, out[0], out[1], out[2], out[3], out[4], None)
    assert e.value.status == 3 and "scratch" in str(e.value)
    ctx.twist_norm_raw_static(x, w, None, None, out[0], out[1], None, None, None, None)      # forward only needs no scratch at any size
    torch.cuda.synchronize()
