"""Full-size checks on the GPU, in the launch configurations bench.py times (Llama-1B-shaped workload: d = 2048,
8 of 16 heads x 128, F' = 2816 of 5632, vocabulary 32000, batch 4 x 2048; Llama-7B-shaped pruned-once workload: d = 4096,
16 of 32 heads x 128, F' = 5504 of 11008, batch 2 x 4096).  The fp64 checker cannot run those shapes
end to end in test time, so the kernels are checked where they can be: sampled entries of every projection
against plain fp64 dot products, sampled heads of the attention kernels against the checker's attention, and a
property of the whole pass (weight gradients computed on the second stream are bit-identical to the serial
schedule)."""
from dataclasses import replace
import math

import numpy as np
import pytest
import torch

import synth_inputs as si
from helpers import rel_fro, to_numpy
from oracle import model as omodel

pytestmark = pytest.mark.gpu

T = 8192
PROJECTIONS = [  # (name, layout, M, N, K) of one layer of the subnet and of the output head
    ("qkv fwd", 0, T, 3072, 2048), ("o fwd", 1, T, 2048, 1024), ("gate/up fwd", 0, T, 5632, 2048), ("down fwd", 1, T, 2048, 2816),
    ("head fwd", 0, T, 32000, 2048), ("qkv dgrad", 1, T, 2048, 3072), ("o dgrad", 0, T, 1024, 2048), ("gate/up dgrad", 1, T, 2048, 5632),
    ("down dgrad", 0, T, 2816, 2048), ("head dgrad", 1, T, 2048, 32000), ("qkv wgrad", 2, 3072, 2048, T), ("o wgrad", 2, 1024, 2048, T),
    ("gate/up wgrad", 2, 5632, 2048, T), ("down wgrad", 2, 2816, 2048, T), ("head wgrad", 2, 32000, 2048, T),
]
# the pruned Llama-7B-shaped layer (d 4096, attention width 2048, F' 5504) and, last two, the longest contractions of the
# unpruned one (down projection over 11008 neurons, gate/up input gradient over 2 x 11008)
PROJECTIONS_7B = [
    ("7b qkv fwd", 0, T, 6144, 4096), ("7b o fwd", 1, T, 4096, 2048), ("7b gate/up fwd", 0, T, 11008, 4096), ("7b down fwd", 1, T, 4096, 5504),
    ("7b head fwd", 0, T, 32000, 4096), ("7b qkv dgrad", 1, T, 4096, 6144), ("7b o dgrad", 0, T, 2048, 4096), ("7b gate/up dgrad", 1, T, 4096, 11008),
    ("7b down dgrad", 0, T, 5504, 4096), ("7b head dgrad", 1, T, 4096, 32000), ("7b qkv wgrad", 2, 6144, 4096, T), ("7b o wgrad", 2, 2048, 4096, T),
    ("7b gate/up wgrad", 2, 11008, 4096, T), ("7b down wgrad", 2, 5504, 4096, T), ("7b head wgrad", 2, 32000, 4096, T),
    ("7b unpruned down fwd", 1, T, 4096, 11008), ("7b unpruned gate/up dgrad", 1, T, 4096, 22016),
]


@pytest.mark.parametrize("name,layout,M,N,K", PROJECTIONS + PROJECTIONS_7B)
def test_projection_at_bench_shape_sampled_entries(lib, name, layout, M, N, K):
    ctx = lib.Context(lib.desc_from_cfg(si.CFG3))
    gen = torch.Generator(device="cuda").manual_seed(M + 3 * N + 7 * K + layout)
    a_shape = (K, M) if layout == 2 else (M, K)
    b_shape = (N, K) if layout == 0 else (K, N)
    A = torch.randn(a_shape, generator=gen, device="cuda").to(torch.bfloat16)
    B = (torch.randn(b_shape, generator=gen, device="cuda") * 0.05).to(torch.bfloat16)
    rng = np.random.default_rng(K)
    # sampled rows and columns: the corners of the output, the last (ragged for N = 32000) tile, and random ones
    rows = np.unique(np.concatenate([[0, 255, 256, M - 1], rng.integers(0, M, 28)]))
    cols = np.unique(np.concatenate([[0, 127, 128, N - 1, N - 2], rng.integers(0, N, 27)]))
    ri, ci = torch.tensor(rows).cuda(), torch.tensor(cols).cuda()
    a_s = to_numpy(A[:, ri].T if layout == 2 else A[ri])                    # [rows, K]
    b_s = to_numpy(B[ci].T if layout == 0 else B[:, ci])                    # [K, cols]
    want = a_s @ b_s
    for out_dtype, tol in ((torch.bfloat16, 5e-3), (torch.float32, 1e-4)):
        out = torch.full((M, N), float("nan"), dtype=out_dtype, device="cuda")
        ctx.twist_gemm_raw(layout, M, N, K, A, B, out)
        torch.cuda.synchronize()
        got = to_numpy(out[ri][:, ci])
        assert rel_fro(got, want) <= tol, (name, out_dtype, rel_fro(got, want))
        assert not torch.isnan(out[-1]).any() and not torch.isnan(out[:, -1]).any()   # the edges were written


@pytest.mark.parametrize("B,N,Hs,picks", [(4, 2048, 8, ((0, 0), (2, 5), (3, 7))), (2, 4096, 16, ((0, 3), (1, 15)))])
def test_attention_at_bench_shape_sampled_heads(lib, B, N, Hs, picks):
    """B = 4, N = 2048, 8 heads of 128 (Llama-1B-shaped subnet) and B = 2, N = 4096, 16 heads (pruned Llama-7B-shaped
    stack): forward output, log-sum-exp and the three input gradients of sampled heads against the checker's attention
    in fp64 on the same bf16 inputs."""
    cfg = si.CFG3
    dh = cfg.d_head
    ctx = lib.Context(lib.desc_from_cfg(cfg))
    gen = torch.Generator(device="cuda").manual_seed(17 + N)
    qkv = torch.randn((B * N, 3 * Hs * dh), generator=gen, device="cuda").to(torch.bfloat16)
    dout = torch.randn((B * N, Hs * dh), generator=gen, device="cuda").to(torch.bfloat16)
    o, lse, dqkv = ctx.twist_attention_raw(qkv, dout, B, N, Hs)
    torch.cuda.synchronize()
    HD = Hs * dh
    for b, h in picks:
        rows = slice(b * N, (b + 1) * N)
        pick = lambda t, part: to_numpy(t[rows, part * HD + h * dh: part * HD + (h + 1) * dh]).reshape(1, N, 1, dh)
        q, k, v = pick(qkv, 0), pick(qkv, 1), pick(qkv, 2)
        do = pick(dout, 0)
        want_o, p = omodel.attention_fwd(q, k, v)
        assert rel_fro(pick(o, 0), want_o) <= 5e-3, (b, h)
        sc = np.einsum("bnhe,bmhe->bhnm", q, k)[0, 0] / math.sqrt(dh)
        sc = np.where(np.triu(np.ones((N, N), dtype=bool), k=1), -np.inf, sc)
        want_lse = np.log(np.exp(sc - sc.max(-1, keepdims=True)).sum(-1)) + sc.max(-1)
        # the kernel normalises by the sum of the probabilities as rounded to bf16: relative 2^-9 / sqrt(#keys) at most
        assert np.abs(to_numpy(lse[b, h]) - want_lse).max() <= 4e-3, (b, h)
        dq, dk, dv = omodel.attention_bwd(p, q, k, v, do)
        for part, want in ((0, dq), (1, dk), (2, dv)):
            err = rel_fro(pick(dqkv, part), want)
            assert err <= 5e-3, (b, h, part, err)


def test_second_stream_weight_gradients_are_bit_identical_to_serial_schedule(lib):
    """Two layers at the benchmark's shape: the pass with the weight-gradient projections on the second stream and
    the pass with every kernel on one stream must give the same bits, and a freshly initialised model's loss sits
    where independent N(0, d 0.02^2) logits put it: ln(vocabulary) + d 0.02^2 / 2."""
    cfg = replace(si.CFG3, n_layers=2, out_unit_major=True)
    S, hs, fs, B, N = 4, 8, 2816, 4, 2048
    gen = torch.Generator(device="cuda").manual_seed(5)
    draw = lambda shp: (torch.ones(shp, device="cuda") if len(shp) == 1 else torch.randn(shp, generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
    layers = [{k: draw(s) for k, s in si.stored_shapes(cfg).items()} for _ in range(cfg.n_layers)]
    globs = {k: draw(s) for k, s in si.global_shapes(cfg).items()}
    fw = lib.FullWeights(layers, globs)
    ctx = lib.Context(lib.desc_from_cfg(cfg))
    plan = ctx.twist_sample(S, hs, fs, seed=3)
    sub = ctx.twist_extract(plan, fw, 1, store=lib.STORE_GRADS)
    ws = torch.empty(ctx.twist_workspace_bytes(sub, B, N), dtype=torch.uint8, device="cuda")
    tok = torch.tensor(si.tokens_zipf(cfg.vocab, B, N, 9)).cuda()
    x, y = tok[:, :-1].contiguous(), tok[:, 1:].contiguous()
    loss = torch.zeros(1, device="cuda")
    results = []
    for overlap in (True, False, True):
        ctx.twist_set_overlap(overlap)
        ctx.twist_subnet_fwd_bwd(sub, x, y, ws, loss)
        torch.cuda.synchronize()
        grads = {(l, k): sub.twist_subnet_view(l, k, 1).clone() for l in range(cfg.n_layers) for k in si.layer_shapes(cfg)}
        grads.update({(-1, k): sub.twist_subnet_view(-1, k, 1).clone() for k in si.global_shapes(cfg)})
        results.append((loss.item(), grads))
    assert abs(results[0][0] - (math.log(cfg.vocab) + cfg.d_model * 0.02 ** 2 / 2)) < 0.2, results[0][0]
    for other in results[1:]:
        assert other[0] == results[0][0]
        for key, g in results[0][1].items():
            if key == (-1, "tok_embed"):
                # rows of repeated tokens are summed with floating-point atomics: the order, hence the last bits, vary
                assert float((g - other[1][key]).norm() / g.norm()) <= 1e-6
            else:
                assert torch.equal(g, other[1][key]), key
            assert torch.isfinite(g).all() and float(g.abs().max()) > 0.0, key
    # The weight gradients above were computed with the token dimension cut into parts (few output tiles, 8192 tokens).
    # The same pass with that disabled (every projection on the 256x256-tile kernel, one contraction) must agree to
    # fp32 summation-order accuracy.
    ctx.twist_set_kernel_choice(gemm_tile=256)
    ctx.twist_subnet_fwd_bwd(sub, x, y, ws, loss)
    torch.cuda.synchronize()
    ctx.twist_set_kernel_choice()
    for l in range(cfg.n_layers):
        for k in ("wq", "wo", "w_gate", "w_down"):
            g0, g1 = results[0][1][(l, k)], sub.twist_subnet_view(l, k, 1)
            assert float((g0 - g1).norm() / g1.norm()) <= 1e-5, (l, k)
