"""Kernel-level parity of the projection kernels (twist_gemm_raw) against the plain matrix product in fp64 on the
same inputs: <= 5e-3 with bf16 operands and output (fp32 accumulation), <= 1e-4 when the output is fp32."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from helpers import rel_fro, to_numpy

pytestmark = pytest.mark.gpu

SHAPES = [  # (M, N, K): several tiles with ragged edges, a tiny one, k not a multiple of the k-tile
    (300, 200, 136), (129, 257, 64), (8, 8, 8), (513, 384, 1000), (256, 256, 4096), (1000, 72, 520), (260, 580, 72),
]


@pytest.mark.parametrize("tile", [128, 256, "plain"])
@pytest.mark.parametrize("layout", [0, 1, 2])
def test_bf16_projection_matches_fp64_product(lib, layout, tile):
    ctx = lib.Context(lib.desc_from_cfg(si.CFG3))
    if tile == "plain":
        ctx.twist_set_kernel_choice(plain_only=True)          # the fall-back kernel for unaligned bf16 operands
    else:
        ctx.twist_set_kernel_choice(gemm_tile=tile)
    for M, N, K in SHAPES:
        a_shape = (K, M) if layout == 2 else (M, K)
        b_shape = (N, K) if layout == 0 else (K, N)
        A = si.to_bf16_grid(si.normal(M + N, f"A{layout}", a_shape))
        B = si.to_bf16_grid(si.normal(K, f"B{layout}", b_shape, 0.05))
        want = (A.T if layout == 2 else A) @ (B.T if layout == 0 else B)
        At, Bt = (torch.tensor(x, dtype=torch.float64).to(torch.bfloat16).cuda() for x in (A, B))
        for out_dtype, tol in ((torch.bfloat16, 5e-3), (torch.float32, 1e-4)):
            out = torch.full((M, N), float("nan"), dtype=out_dtype, device="cuda")
            guard = torch.zeros(64, dtype=out_dtype, device="cuda")       # allocated right after: must stay zero
            ctx.twist_gemm_raw(layout, M, N, K, At, Bt, out, alpha=0.5)
            torch.cuda.synchronize()
            assert rel_fro(to_numpy(out), 0.5 * want) <= tol, (layout, tile, M, N, K, out_dtype)
            assert not guard.any()


def test_fp32_projection(lib):
    ctx = lib.Context(lib.desc_from_cfg(si.CFG1))
    for layout in (0, 1, 2):
        M, N, K = 150, 70, 90
        a_shape = (K, M) if layout == 2 else (M, K)
        b_shape = (N, K) if layout == 0 else (K, N)
        A, B = si.normal(1, "a", a_shape), si.normal(2, "b", b_shape)
        A, B = A.astype(np.float32).astype(np.float64), B.astype(np.float32).astype(np.float64)
        want = (A.T if layout == 2 else A) @ (B.T if layout == 0 else B)
        out = torch.empty((M, N), dtype=torch.float32, device="cuda")
        ctx.twist_gemm_raw(layout, M, N, K, torch.tensor(A, dtype=torch.float32).cuda(), torch.tensor(B, dtype=torch.float32).cuda(), out)
        assert rel_fro(to_numpy(out), want) <= 1e-4


def test_raw_rejects_bad_strides(lib):
    ctx = lib.Context(lib.desc_from_cfg(si.CFG3))
    A = torch.zeros(16, 8, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(16, 16, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(lib.TwistError):
        ctx.twist_gemm_raw(0, 16, 16, 32, A, A, out)      # K larger than the row stride
    with pytest.raises(lib.TwistError):
        ctx.twist_set_kernel_choice(gemm_tile=64)         # only 0, 128 and 256 exist
