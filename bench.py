#!/usr/bin/env python3
"""Benchmark of the TwIST hot path on one MI355X.

One "step" is one whole training round of the Llama-1B-shaped workload: sample (Algorithm 1) -> extract S=4
overlapping half-width subnets -> per subnet `--local-steps` x (forward+backward + AdamW) -> aggregate.
`value` is the whole-job token throughput of that round (every phase inside the timed region, inputs and
weights resident in HBM).  Alongside: the forward+backward-only token rate, the extract / aggregate GB/s at
the Llama-7B stack shape, the roofline figures of the dominant kernels and the CPU checker timed on the host.

Prints ONE JSON line on stdout.  Everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from dataclasses import replace

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def device_weights(cfg, seed, si, torch):
    """bf16 N(0, 0.02) weights drawn on the device (norm gains 1), in the library's tensor naming."""
    gen = torch.Generator(device="cuda").manual_seed(seed)

    def draw(name, shp):
        if len(shp) == 1:
            return torch.ones(shp, dtype=torch.bfloat16, device="cuda") if name.endswith("_w") else torch.zeros(shp, dtype=torch.bfloat16, device="cuda")
        out = torch.empty(shp, dtype=torch.bfloat16, device="cuda")
        rows = max(1, (1 << 24) // shp[1])
        for r in range(0, shp[0], rows):                       # chunked: no fp32 copy of a whole matrix
            n = min(rows, shp[0] - r)
            out[r:r + n] = (torch.randn((n, shp[1]), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
        return out

    layers = [{k: draw(k, s) for k, s in si.stored_shapes(cfg).items()} for _ in range(cfg.n_layers)]
    globs = {k: draw(k, s) for k, s in si.global_shapes(cfg).items()}
    return layers, globs


def flops_fwd_bwd(cfg, hs, F, B, N):
    """Algorithmic FLOPs of one forward+backward of the subnet: 3 x forward; 2MNK per projection; causal
    attention counted at half of 4 B H' N^2 d_head."""
    T, d, hd = B * N, cfg.d_model, hs * cfg.d_head
    nf = 2 if cfg.act == "swiglu" else 1
    per_layer = 2 * T * d * 3 * hd + 2 * T * hd * d + 2 * T * d * nf * F + 2 * T * F * d + 0.5 * 4 * B * hs * N * N * cfg.d_head
    head = 2 * T * d * cfg.vocab
    return 3 * (cfg.n_layers * per_layer + head)


# HBM-side bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this benchmark's own command and
# calibrated against streaming kernels of known size in the same run (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0; the counter
# sits behind the L2, so reads served by the Infinity Cache are included).  Source: profiles/bench_hbm_traffic_fetch_write.txt
TRAFFIC_PROJECTION_LAUNCH = 316.7e6         # average over every projection launch of a forward+backward pass
TRAFFIC_EXTRACT_LAYER_LAUNCH = 405.2e6      # one layer of one subnet at the 7B shape, unit-major layout
TRAFFIC_AGGREGATE_LAYER_LAUNCH = 2029.6e6   # one layer, 8 subnets


def bytes_fwd_bwd_projections(cfg, hs, F, B, N):
    """Algorithmic bytes of the projection launches of one forward+backward: each operand read once, the output
    written once (fp32 residual read and written where the epilogue adds it), and their number."""
    T, d, hd, V = B * N, cfg.d_model, hs * cfg.d_head, cfg.vocab
    nf = 2 if cfg.act == "swiglu" else 1
    def g(m, n, k, out_b, resid=False):
        return 2 * (m * k + k * n) + out_b * m * n + (4 * m * n if resid else 0)
    per_layer = (g(T, 3 * hd, d, 2) + g(T, d, hd, 4, True) + g(T, nf * F, d, 2) + g(T, d, F, 4, True)        # forward
                 + g(T, d, 3 * hd, 2) + g(T, hd, d, 2) + g(T, d, nf * F, 2) + g(T, F, d, 2)                    # input gradients
                 + g(3 * hd, d, T, 4) + g(hd, d, T, 4) + g(nf * F, d, T, 4) + g(F, d, T, 4))                  # weight gradients
    head = g(T, V, d, 2) + g(T, d, V, 2) + g(V, d, T, 4)
    return cfg.n_layers * per_layer + head, cfg.n_layers * 12 + 3


def bench_train(args, tw, si, torch):
    cfg = replace(si.CFG3, out_unit_major=True)      # output projections stored unit-major: every gather is a row gather
    S, hs, fs, B, N = 4, 8, 2816, 4, 2048
    log(f"[bench] workload llama1b_round: L={cfg.n_layers} d={cfg.d_model} H'={hs} F'={fs} S={S} B={B} N={N} local_steps={args.local_steps}")
    layers, globs = device_weights(cfg, 0, si, torch)
    fw = tw.FullWeights(layers, globs)
    ctx = tw.Context(tw.desc_from_cfg(cfg))
    ctx.twist_set_overlap(not args.no_overlap)
    plan0 = ctx.twist_sample(S, hs, fs, seed=0, rnd=0)
    nbytes = ctx.twist_subnet_bytes(plan0, tw.STORE_ADAMW)
    stor = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(S)]
    sub0 = ctx.twist_extract(plan0, fw, 0, store=tw.STORE_ADAMW, storage=stor[0])
    ws = torch.empty(ctx.twist_workspace_bytes(sub0, B, N), dtype=torch.uint8, device="cuda")
    sub0.close(); plan0.close()
    log(f"[bench] subnet storage {nbytes / 2**30:.2f} GiB x {S}, workspace {ws.numel() / 2**30:.2f} GiB")
    # Zipf(1.1) token streams, a different one per subnet and local step
    n_streams = S * args.local_steps
    toks = [torch.tensor(si.tokens_zipf(cfg.vocab, B, N, 100 + i)).cuda() for i in range(n_streams)]
    xs = [t[:, :-1].contiguous() for t in toks]
    ys = [t[:, 1:].contiguous() for t in toks]
    loss = torch.zeros(1, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)
    phase_ms = {"sample": 0.0, "extract": 0.0, "fwd_bwd": 0.0, "opt_step": 0.0, "aggregate": 0.0}
    fb_each = []   # each timed forward+backward launch, ms

    def one_round(rnd, timed):
        marks = []
        t0 = time.perf_counter()
        plan = ctx.twist_sample(S, hs, fs, seed=0, rnd=rnd)
        t_sample = (time.perf_counter() - t0) * 1e3
        e0 = ev(); e0.record()
        subs = ctx.twist_extract_all(plan, fw, store=tw.STORE_ADAMW, storages=stor)   # the S subnets are resident together: one pass
        e1 = ev(); e1.record()
        marks.append(("extract", e0, e1))
        for s, sub in enumerate(subs):
            for it in range(args.local_steps):
                i = s * args.local_steps + it
                a = ev(); a.record()
                ctx.twist_subnet_fwd_bwd(sub, xs[i], ys[i], ws, loss)
                b = ev(); b.record()
                ctx.twist_subnet_step(sub, tw.OPT_ADAMW, lr=1e-4, weight_decay=0.01)
                c = ev(); c.record()
                marks.append(("fwd_bwd", a, b)); marks.append(("opt_step", b, c))
        a = ev(); a.record()
        ctx.twist_aggregate(plan, subs, fw)
        b = ev(); b.record()
        marks.append(("aggregate", a, b))
        torch.cuda.synchronize()
        if timed:
            phase_ms["sample"] += t_sample
            for k, x, y in marks:
                t = x.elapsed_time(y)
                phase_ms[k] += t
                if k == "fwd_bwd":
                    fb_each.append(t)
        for sub in subs:
            sub.close()
        plan.close()

    for w in range(args.warmup):
        one_round(w, False)
        log(f"[bench] warmup round {w} done, loss {loss.item():.4f}")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_round(args.warmup + k, True)
        log(f"[bench] timed round {k} done, loss {loss.item():.4f}")
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # Per-launch durations of the projection kernel: one more forward+backward per subnet with every kernel on
    # one stream (in the timed region the weight-gradient projections overlap other kernels on a second stream,
    # where a launch's own duration says little), each launch bracketed by HIP events on that stream.
    plan = ctx.twist_sample(S, hs, fs, seed=0, rnd=args.warmup + args.steps)
    subs = ctx.twist_extract_all(plan, fw, store=tw.STORE_ADAMW, storages=stor)
    ctx.twist_set_overlap(False)
    ctx.twist_subnet_fwd_bwd(subs[0], xs[0], ys[0], ws, loss)
    ctx.twist_profile_gemm(True)
    for s, sub in enumerate(subs):
        ctx.twist_subnet_fwd_bwd(sub, xs[s * args.local_steps], ys[s * args.local_steps], ws, loss)
    n_gemm, gemm_ms, gemm_flops = ctx.twist_profile_gemm_read()
    ctx.twist_profile_gemm(False)
    ctx.twist_set_overlap(not args.no_overlap)
    for sub in subs:
        sub.close()
    plan.close()
    tokens = args.steps * S * args.local_steps * B * N
    fb_calls = args.steps * S * args.local_steps
    fb_ms = phase_ms["fwd_bwd"] / fb_calls
    alg = flops_fwd_bwd(cfg, hs, fs, B, N)
    res = {
        "tokens_per_s": tokens / dt, "ms_per_step": dt * 1e3 / args.steps,
        "fwd_bwd_ms": fb_ms, "fwd_bwd_median_ms": sorted(fb_each)[len(fb_each) // 2], "fwd_bwd_min_ms": min(fb_each), "fwd_bwd_timed_calls": len(fb_each),
        "fwd_bwd_tokens_per_s": B * N / (fb_ms * 1e-3),
        "fwd_bwd_tflops": alg / (fb_ms * 1e-3) / 1e12, "fwd_bwd_frac_mfma_peak": alg / (fb_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "phase_ms_per_step": {k: v / args.steps for k, v in phase_ms.items()},
        "gemm": {"launches": n_gemm, "avg_ms": gemm_ms / max(n_gemm, 1), "tflops": gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms else 0.0,
                 "flops_per_launch": gemm_flops / max(n_gemm, 1)},
        "loss": loss.item(),
    }
    pb, pn = bytes_fwd_bwd_projections(cfg, hs, fs, B, N)
    res["gemm"]["algorithmic_bytes_per_launch"] = pb / pn
    if args.native_round:
        # the same round through twist_round: the loop runs inside the library, ONE subnet is resident at a time and the
        # aggregation is the running fp32 sum (Section 3's round with the repartition interval of Section 5)
        optd = {"kind": tw.OPT_ADAMW, "lr": 1e-4, "weight_decay": 0.01}
        sb, wb, ib = ctx.twist_round_bytes(S, hs, fs, B, N, args.local_steps, opt=optd)
        image = torch.empty(ib, dtype=torch.uint8, device="cuda")
        x_all = torch.stack(xs).view(S, args.local_steps, B, N).contiguous()
        y_all = torch.stack(ys).view(S, args.local_steps, B, N).contiguous()
        losses = torch.zeros(S, args.local_steps, device="cuda")
        ctx.twist_round(fw, x_all, y_all, S, hs, fs, stor[0], ws, image, losses, seed=0, rnd=100, opt=optd)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for r in range(args.steps):
            ctx.twist_round(fw, x_all, y_all, S, hs, fs, stor[0], ws, image, losses, seed=0, rnd=101 + r, opt=optd)
        torch.cuda.synchronize()
        dtn = time.perf_counter() - t0
        res["native_round"] = {"tokens_per_s": tokens / dtn, "ms_per_round": dtn * 1e3 / args.steps, "resident_subnets": 1,
                               "running_sum_image_GiB": ib / 2**30, "last_loss": float(losses[-1, -1])}
        del image
    del stor, ws, layers, globs, fw
    torch.cuda.empty_cache()
    return res


def bench_movers(args, tw, si, torch, unit_major=True):
    """extract x8 and aggregate at the Llama-7B layer-stack shape (memory-bound)."""
    cfg = replace(si.CFG4, out_unit_major=unit_major)
    S, hs, fs = 8, 16, 5504
    layers, _ = device_weights(cfg, 1, si, torch)
    fw = tw.FullWeights(layers)
    ctx = tw.Context(tw.desc_from_cfg(cfg))
    t_sample = []
    for r in range(4):   # host time of Algorithm 1 + table upload at this shape (first call untimed)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plan = ctx.twist_sample(S, hs, fs, seed=11, rnd=r)
        t_sample.append((time.perf_counter() - t0) * 1e3)
        plan.close()
    plan = ctx.twist_sample(S, hs, fs, seed=11)
    nb = ctx.twist_subnet_bytes(plan)
    stor = [torch.empty(nb, dtype=torch.uint8, device="cuda") for _ in range(S)]
    part = sum(v.numel() for v in layers[0].values() if v.dim() == 2) * cfg.n_layers
    shared = sum(v.numel() for v in layers[0].values() if v.dim() == 1) * cfg.n_layers
    kept = part // 2
    ex_bytes = 2 * 2 * (kept + shared) * S                 # read kept + write kept, bf16
    ag_bytes = 2 * (S * (kept + shared) + part + shared)   # read every subnet element + write every central element
    gen = torch.Generator(device="cuda").manual_seed(7)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    ex_ms, ag_ms, rs_ms, xa_ms = [], [], [], []
    image = torch.empty(ctx.twist_aggregate_image_bytes(), dtype=torch.uint8, device="cuda")
    # running-sum form: per added element read 2 B + write 4 B (+ read 4 B unless first owner); finish reads 4 B, writes 2 B
    rs_bytes = (2 + 4) * S * (kept + shared) + 4 * (S * (kept + shared) - (part + shared)) + (4 + 2) * (part + shared)
    warm, reps = 3, args.mover_reps
    for it in range(warm + reps):
        a = ev(); a.record()
        subs = [ctx.twist_extract(plan, fw, s, storage=stor[s]) for s in range(S)]
        b = ev(); b.record()
        # stand-in for local training (not timed): perturb the subnet weights by N(0, 1e-3), in chunks
        for st in stor:
            v = st.view(torch.bfloat16)
            for o in range(0, v.numel(), 1 << 26):
                c = v[o:o + (1 << 26)]
                c.add_((torch.randn(c.shape, generator=gen, device="cuda") * 1e-3).to(torch.bfloat16))
        c0 = ev(); c0.record()
        ctx.twist_aggregate(plan, subs, fw)
        d = ev(); d.record()
        f0 = ev(); f0.record()
        subs_all = ctx.twist_extract_all(plan, fw, storages=stor)   # all 8 subnets in one pass over the central model
        f1 = ev(); f1.record()
        acc = ctx.twist_aggregate_begin(plan, image)      # the same aggregation, one subnet at a time
        for sub in subs:
            acc.twist_aggregate_add(sub)
        acc.twist_aggregate_finish(fw)
        e = ev(); e.record()
        torch.cuda.synchronize()
        acc.close()
        for sb in subs_all:
            sb.close()
        if it >= warm:
            xa_ms.append(f0.elapsed_time(f1))
            ex_ms.append(a.elapsed_time(b)); ag_ms.append(c0.elapsed_time(d)); rs_ms.append(d.elapsed_time(e))
    med = lambda v: sorted(v)[len(v) // 2]
    res = {"extract_ms": med(ex_ms), "aggregate_ms": med(ag_ms), "extract_GBps": ex_bytes / med(ex_ms) / 1e6, "aggregate_GBps": ag_bytes / med(ag_ms) / 1e6,
           "extract_alg_GB": ex_bytes / 1e9, "aggregate_alg_GB": ag_bytes / 1e9,
           # one pass for all subnets: reads the central model once (not once per subnet), writes the same bytes
           "extract_all_ms": med(xa_ms), "extract_all_GBps_on_per_subnet_bytes": ex_bytes / med(xa_ms) / 1e6,
           "extract_all_moved_GB": (2 * (part + shared) + 2 * (kept + shared) * S) / 1e9,
           "extract_all_GBps_moved": (2 * (part + shared) + 2 * (kept + shared) * S) / med(xa_ms) / 1e6,
           "running_sum_aggregate_ms": med(rs_ms), "running_sum_aggregate_GBps": rs_bytes / med(rs_ms) / 1e6, "running_sum_alg_GB": rs_bytes / 1e9,
           "sample_host_ms": sorted(t_sample[1:])[1],
           "layers": cfg.n_layers, "subnets": S, "layers_per_launch": "as many whole layers as fit the library's 44-entry job table (4 at this shape)", "warmup": warm, "timed_reps": reps,
           "extract_min_ms": min(ex_ms), "aggregate_min_ms": min(ag_ms), "extract_all_min_ms": min(xa_ms), "running_sum_aggregate_min_ms": min(rs_ms),
           "extract_frac_hbm_peak": ex_bytes / med(ex_ms) / 1e6 / PEAK_HBM_GBS, "aggregate_frac_hbm_peak": ag_bytes / med(ag_ms) / 1e6 / PEAK_HBM_GBS}
    # plain device copy of known size, the practical ceiling the fractions should be read against
    x = torch.empty(4 << 30, dtype=torch.uint8, device="cuda"); y = torch.empty_like(x)
    for _ in range(2):
        y.copy_(x)
    a = ev(); a.record()
    for _ in range(5):
        y.copy_(x)
    b = ev(); b.record(); torch.cuda.synchronize()
    res["copy_ceiling_GBps"] = 2 * x.numel() * 5 / a.elapsed_time(b) / 1e6
    del x, y, stor, layers, fw, image
    torch.cuda.empty_cache()
    return res


def bench_golden_ticket(args, tw, si, torch):
    """configs[4]: forward+backward of the Llama-7B-shaped stack pruned once to 16 of 32 heads and 5504 of 11008
    neurons per layer (deployment extract, untimed), next to the unpruned stack at the same batch 2 x 4096."""
    cfg = replace(si.CFG5, out_unit_major=True)
    B, N = 2, 4096
    layers, globs = device_weights(cfg, 2, si, torch)
    fw = tw.FullWeights(layers, globs)
    ctx = tw.Context(tw.desc_from_cfg(cfg))
    tok = torch.randint(0, cfg.vocab, (B, N + 1), generator=torch.Generator(device="cuda").manual_seed(3), device="cuda", dtype=torch.int32)
    x, y = tok[:, :-1].contiguous(), tok[:, 1:].contiguous()
    loss = torch.zeros(1, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)
    res = {}
    for tag, hs, fs in (("pruned", 16, 5504), ("unpruned", 32, 11008)):
        plan = ctx.twist_sample(1, hs, fs, seed=5, require_coverage=False)
        sub = ctx.twist_extract(plan, fw, 0, store=tw.STORE_GRADS)
        ws = torch.empty(ctx.twist_workspace_bytes(sub, B, N), dtype=torch.uint8, device="cuda")
        ctx.twist_subnet_fwd_bwd(sub, x, y, ws, loss)
        a = ev(); a.record()
        reps = 3
        for _ in range(reps):
            ctx.twist_subnet_fwd_bwd(sub, x, y, ws, loss)
        b = ev(); b.record(); torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        fl = flops_fwd_bwd(cfg, hs, fs, B, N)
        res[tag] = {"fwd_bwd_ms": ms, "tokens_per_s": B * N / (ms * 1e-3), "tflops": fl / (ms * 1e-3) / 1e12,
                    "frac_mfma_peak": fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, "loss": loss.item()}
        sub.close(); plan.close()
        del ws, sub
        torch.cuda.empty_cache()
    res["speedup_pruned_over_unpruned"] = res["unpruned"]["fwd_bwd_ms"] / res["pruned"]["fwd_bwd_ms"]
    res["ideal_flop_ratio"] = flops_fwd_bwd(cfg, 32, 11008, B, N) / flops_fwd_bwd(cfg, 16, 5504, B, N)
    return res


def bench_mfma_ceiling(tw, si, torch):
    """The bf16 matrix instruction alone on the whole chip (no loads, about half a second per setting so that the clock
    settles where the power limit puts it): the ceiling for any kernel built on it, next to the published 2.5 PFLOP/s."""
    ctx = tw.Context(tw.desc_from_cfg(si.CFG3))
    out = {}
    for tag, rnd in (("constant_operands", False), ("random_operands", True)):
        for wps in (1, 2):
            ctx.twist_profile_mfma_ceiling(wps, 200000, rnd)
            out[f"{tag}_{wps}_waves_per_simd_tflops"] = ctx.twist_profile_mfma_ceiling(wps, 3000000 // wps, rnd)
    best = max(v for k, v in out.items() if k.startswith("random"))
    out.update({"instruction": "v_mfma_f32_32x32x16_bf16, 4 independent accumulator tiles per wave, operands in registers, about 0.5 s per setting",
                "random_operands_best_tflops": best, "random_operands_frac_of_published_peak": best / PEAK_BF16_TFLOPS})
    return out


def bench_gpt2_small(args, tw, si, torch):
    """configs[1]: GPT-2-small-shaped model (12 layers, d 768, 12 heads, d_ff 3072, vocabulary 50257, tied head), S = 4
    subnets of 3 heads and a disjoint quarter of the neurons each, batch 8 x 1024 uniform tokens: extract, one
    forward+backward per subnet back to back, aggregate."""
    cfg = replace(si.CFG2, out_unit_major=True)
    S, hs, fs, B, N = 4, 3, 768, 8, 1024
    layers, globs = device_weights(cfg, 8, si, torch)
    fw = tw.FullWeights(layers, globs)
    ctx = tw.Context(tw.desc_from_cfg(cfg))
    plan = ctx.twist_sample(S, hs, fs, seed=2)
    nb = ctx.twist_subnet_bytes(plan, tw.STORE_GRADS)
    stor = [torch.empty(nb, dtype=torch.uint8, device="cuda") for _ in range(S)]
    gen = torch.Generator(device="cuda").manual_seed(9)
    toks = [torch.randint(0, cfg.vocab, (B, N + 1), generator=gen, device="cuda", dtype=torch.int32) for _ in range(S)]
    xs, ys = [t[:, :-1].contiguous() for t in toks], [t[:, 1:].contiguous() for t in toks]
    loss = torch.zeros(1, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)
    ws = None
    t_ex, t_fb, t_ag = [], [], []
    for it in range(2 + 5):
        a = ev(); a.record()
        subs = ctx.twist_extract_all(plan, fw, store=tw.STORE_GRADS, storages=stor)
        b = ev(); b.record()
        if ws is None:
            ws = torch.empty(ctx.twist_workspace_bytes(subs[0], B, N), dtype=torch.uint8, device="cuda")
        for s, sub in enumerate(subs):
            ctx.twist_subnet_fwd_bwd(sub, xs[s], ys[s], ws, loss)
        c = ev(); c.record()
        ctx.twist_aggregate(plan, subs, fw)
        d = ev(); d.record(); torch.cuda.synchronize()
        if it >= 2:
            t_ex.append(a.elapsed_time(b)); t_fb.append(b.elapsed_time(c)); t_ag.append(c.elapsed_time(d))
        for sub in subs:
            sub.close()
    med = lambda v: sorted(v)[len(v) // 2]
    fl = flops_fwd_bwd(cfg, hs, fs, B, N)
    fb = med(t_fb) / S
    res = {"extract_all_ms": med(t_ex), "fwd_bwd_x4_ms": med(t_fb), "aggregate_ms": med(t_ag), "fwd_bwd_ms_per_subnet": fb,
           "fwd_bwd_tokens_per_s": B * N / (fb * 1e-3), "fwd_bwd_tflops": fl / (fb * 1e-3) / 1e12,
           "fwd_bwd_frac_mfma_peak": fl / (fb * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
           "whole_pass_tokens_per_s": S * B * N / ((med(t_ex) + med(t_fb) + med(t_ag)) * 1e-3), "loss": loss.item(),
           "workload": "configs[1]: S=4 disjoint quarter-width subnets (3 of 12 heads, 768 of 3072 neurons), batch 8x1024, tied 50257-token head"}
    plan.close()
    del stor, ws, layers, globs, fw
    torch.cuda.empty_cache()
    return res


def bench_clock_under_load(tw, si, torch):
    """Shader clock reported by rocm-smi while the projection kernel runs back to back on the whole chip (8192^3, about
    3 s), next to the idle reading: the published MFMA peak assumes the 2.4 GHz boost clock, the chip holds less under
    this load.  Best effort: None when rocm-smi is missing or prints something else."""
    import re
    import subprocess
    import threading

    def sclk():
        try:
            r = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=20)
            m = re.search(r"sclk clock level: \S+ \((\d+)Mhz\)", r.stdout)
            return int(m.group(1)) if m else None
        except Exception:
            return None

    idle = sclk()
    if idle is None:
        return None
    ctx = tw.Context(tw.desc_from_cfg(si.CFG3))
    g = torch.Generator(device="cuda").manual_seed(1)
    n = 8192
    a = torch.randn(n, n, device="cuda", generator=g).bfloat16()
    b = torch.randn(n, n, device="cuda", generator=g).bfloat16()
    c = torch.empty(n, n, device="cuda", dtype=torch.bfloat16)
    samples = []

    def sampler():
        time.sleep(1.5)
        for _ in range(2):
            samples.append(sclk())
            time.sleep(0.4)

    th = threading.Thread(target=sampler)
    th.start()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0, launches = time.time(), 0
    e0.record()
    while time.time() - t0 < 3.0:
        for _ in range(50):
            ctx.twist_gemm_raw(0, n, n, n, a, b, c)
        torch.cuda.synchronize()
        launches += 50
    e1.record()
    torch.cuda.synchronize()
    th.join()
    samples = [x for x in samples if x]
    if not samples:
        return None
    mhz = sum(samples) / len(samples)
    tf = 2.0 * n ** 3 * launches / e0.elapsed_time(e1) / 1e9
    return {"before_mhz": idle, "projection_load_mhz": mhz, "projection_8192_cubed_tflops": tf,
            "mfma_peak_at_that_clock_tflops": PEAK_BF16_TFLOPS * mhz / 2400.0, "frac_of_peak_at_that_clock": tf / (PEAK_BF16_TFLOPS * mhz / 2400.0)}


def bench_latency_ablation(args, tw, si, torch):
    """Latency study of Section 5 (Figure 4 / Table 2) on synthetic data: GPT-2-small shape, blocks = heads and
    d_ff/12-neuron FFN blocks, first and last two layers shared, kept blocks kappa in {10, 8, 6, 4} of 12 for the
    attention blocks, the FFN blocks, or both; milliseconds per batch of 2 x 1024 tokens for forward+backward+AdamW
    on one subnet, next to the full-width model."""
    cfg = replace(si.CFG2, ffn_granule=si.CFG2.d_ff // 12)
    B, N = 2, 1024
    layers, globs = device_weights(cfg, 4, si, torch)
    fw = tw.FullWeights(layers, globs)
    ctx = tw.Context(tw.desc_from_cfg(cfg))
    shared = [1, 1] + [0] * (cfg.n_layers - 4) + [1, 1]
    tok = torch.randint(0, cfg.vocab, (B, N + 1), generator=torch.Generator(device="cuda").manual_seed(6), device="cuda", dtype=torch.int32)
    x, y = tok[:, :-1].contiguous(), tok[:, 1:].contiguous()
    loss = torch.zeros(1, device="cuda")
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def ms_per_batch(heads, ffn):
        plan = ctx.twist_sample(3, heads, ffn, seed=1, layer_shared=shared, require_coverage=heads * 3 >= 12 and ffn * 3 >= 12)
        sub = ctx.twist_extract(plan, fw, 0, store=tw.STORE_ADAMW)
        ws = torch.empty(ctx.twist_workspace_bytes(sub, B, N), dtype=torch.uint8, device="cuda")
        for _ in range(2):
            ctx.twist_subnet_fwd_bwd(sub, x, y, ws, loss)
            ctx.twist_subnet_step(sub, tw.OPT_ADAMW, lr=1e-4)
        a = ev(); a.record()
        reps = 10
        for _ in range(reps):
            ctx.twist_subnet_fwd_bwd(sub, x, y, ws, loss)
            ctx.twist_subnet_step(sub, tw.OPT_ADAMW, lr=1e-4)
        b = ev(); b.record()
        for _ in range(reps):                       # deployment use of the same subnet: forward only (Section 4.2)
            ctx.twist_subnet_forward(sub, x, y, ws, loss)
        c = ev(); c.record(); torch.cuda.synchronize()
        sub.close(); plan.close()
        return a.elapsed_time(b) / reps, b.elapsed_time(c) / reps

    full = ms_per_batch(12, 12)
    res = {"batch": [B, N], "full_width_ms": full[0], "full_width_forward_ms": full[1]}
    for k in (10, 8, 6, 4):
        at, ff, bo = ms_per_batch(k, 12), ms_per_batch(12, k), ms_per_batch(k, k)
        res[f"kappa_{k}"] = {"attn_ms": at[0], "ffn_ms": ff[0], "both_ms": bo[0],
                             "attn_forward_ms": at[1], "ffn_forward_ms": ff[1], "both_forward_ms": bo[1]}
    return res


def cpu_baseline(si):
    """The CPU checker as it stands, timed on a bounded sample of the same workload: the Llama-1B-shaped
    half-width subnet at full widths and vocabulary with 1 and 2 layers on 2 x 1024 tokens; the per-layer
    and the embedding/head costs are separated and extrapolated to the 22-layer model."""
    import numpy as np
    from oracle import model as omodel, move as omove
    from oracle.sample import sample_plan
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    B, N = 2, 1024
    times = {}
    for L in (1, 2):
        cfg = replace(si.CFG3, n_layers=L)
        full = si.make_weights(cfg, 0)
        plan = sample_plan(L, cfg.n_heads, cfg.n_ffn_units, 4, 8, 2816, 0)
        sub = omove.extract(full, plan, 0, cfg.d_head)
        t = si.tokens_zipf(cfg.vocab, B, N, 5)
        t0 = time.perf_counter()
        omodel.forward_backward(cfg, sub, t[:, :-1], t[:, 1:])
        times[L] = time.perf_counter() - t0
    per_layer = max(times[2] - times[1], 1e-9)
    full_time = times[1] + 21 * per_layer
    return {"value": B * N / full_time, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fp64 numpy checker, forward+backward of the Llama-1B-shaped half-width subnet on {B}x{N} tokens, measured with 1 and 2 layers "
                      f"({times[1]:.2f} s, {times[2]:.2f} s) and extrapolated to 22 layers"}


def cpu_baseline_one_thread(si):
    """The same checker held to ONE thread, on a smaller bounded sample (1 x 256 tokens, 1 and 2 layers at the
    Llama-1B-shaped half-width subnet's widths and vocabulary), extrapolated to 22 layers the same way."""
    from oracle import model as omodel, move as omove
    from oracle.sample import sample_plan
    from threadpoolctl import threadpool_limits
    B, N = 1, 256
    times = {}
    with threadpool_limits(limits=1):
        for L in (1, 2):
            cfg = replace(si.CFG3, n_layers=L)
            full = si.make_weights(cfg, 0)
            plan = sample_plan(L, cfg.n_heads, cfg.n_ffn_units, 4, 8, 2816, 0)
            sub = omove.extract(full, plan, 0, cfg.d_head)
            t = si.tokens_zipf(cfg.vocab, B, N, 5)
            t0 = time.perf_counter()
            omodel.forward_backward(cfg, sub, t[:, :-1], t[:, 1:])
            times[L] = time.perf_counter() - t0
    per_layer = max(times[2] - times[1], 1e-9)
    return {"value": B * N / (times[1] + 21 * per_layer), "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": f"fp64 numpy checker on one thread, forward+backward of the Llama-1B-shaped half-width subnet on {B}x{N} tokens, measured with 1 "
                      f"and 2 layers ({times[1]:.2f} s, {times[2]:.2f} s) and extrapolated to 22 layers"}


def cpu_baseline_movers(si):
    """The CPU checker's extract and aggregate on a bounded sample of the mover workload: ONE Llama-7B-shaped layer at a
    quarter of its width (d_model 4096, 8 of 32 heads, d_ff 2752 of 11008: same row lengths, a quarter of the rows),
    S=8 half-width subnets.  GB/s is quoted on the workload's own algorithmic bytes (2-byte elements), like the GPU's."""
    import numpy as np
    from oracle import move as omove
    from oracle.sample import sample_plan
    cfg = replace(si.CFG4, n_layers=1, n_heads=8, d_ff=2752)
    S, hs, fs = 8, 4, 1376
    full = si.make_weights(cfg, 0)
    plan = sample_plan(1, cfg.n_heads, cfg.n_ffn_units, S, hs, fs, 0)
    t0 = time.perf_counter()
    subs = [omove.extract(full, plan, s, cfg.d_head) for s in range(S)]
    t_ex = time.perf_counter() - t0
    t0 = time.perf_counter()
    omove.aggregate(full, plan, subs, cfg.d_head)
    t_ag = time.perf_counter() - t0
    n_full = sum(v.size for v in full["layers"][0].values())
    n_sub = sum(v.size for v in subs[0]["layers"][0].values())
    ex_bytes, ag_bytes = 2 * 2 * n_sub * S, 2 * (S * n_sub + n_full)
    return {"value": (ex_bytes + ag_bytes) / (t_ex + t_ag) / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "extract_GBps": ex_bytes / t_ex / 1e9, "aggregate_GBps": ag_bytes / t_ag / 1e9,
            "sample": f"fp64 numpy checker, extract x{S} ({t_ex:.1f} s) and aggregate ({t_ag:.1f} s) of one Llama-7B-shaped layer at quarter "
                      "width (8 heads, d_ff 2752), bytes counted as 2-byte elements"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--local-steps", type=int, default=10, help="AdamW steps per subnet per round")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--skip-movers", action="store_true")
    ap.add_argument("--mover-reps", type=int, default=10, help="timed repetitions of the movers leg (after 3 warm-up ones)")
    ap.add_argument("--skip-golden", action="store_true", help="skip the pruned-versus-unpruned 7B-shaped forward+backward leg")
    ap.add_argument("--native-round", action="store_true", help="also time the same round through twist_round (library-side loop, one subnet resident)")
    ap.add_argument("--skip-clock", action="store_true", help="skip the rocm-smi clock reading under projection load")
    ap.add_argument("--skip-ablation", action="store_true", help="skip the GPT-2-small-shaped latency study (kept blocks 10/8/6/4 of 12)")
    ap.add_argument("--skip-gpt2", action="store_true", help="skip the GPT-2-small-shaped leg (4 x forward+backward at 8 x 1024, then aggregate)")
    ap.add_argument("--no-overlap", action="store_true", help="keep every kernel on one stream also in the timed region (for per-kernel profiles)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the S subnets run back-to-back on it); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2511_03983_amd as tw          # raises if the HIP library is missing: no fallback
    import synth_inputs as si
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    train = bench_train(args, tw, si, torch)
    log("[bench] train:", json.dumps(train))
    movers = None if args.skip_movers else bench_movers(args, tw, si, torch, unit_major=True)
    log("[bench] movers (unit-major output projections):", json.dumps(movers))
    movers_rm = None if args.skip_movers else bench_movers(args, tw, si, torch, unit_major=False)
    log("[bench] movers ([out, in] output projections):", json.dumps(movers_rm))
    golden = None if args.skip_golden else bench_golden_ticket(args, tw, si, torch)
    log("[bench] golden ticket (7B shape, pruned vs unpruned):", json.dumps(golden))
    # (not under a profiler: its preloaded library makes every child process a GPU process, and rocm-smi is a script
    # whose interpreter hop such a process may not take on the boxes this runs on)
    profiled = any("rocprof" in os.environ.get(k, "").lower() for k in ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES", "HSA_TOOLS_LIB")) or \
        any(k.startswith("ROCPROF") for k in os.environ)
    clock = None if (args.skip_movers or args.skip_clock or profiled) else bench_clock_under_load(tw, si, torch)
    log("[bench] clock under projection load:", json.dumps(clock))
    gpt2 = None if args.skip_gpt2 else bench_gpt2_small(args, tw, si, torch)
    log("[bench] GPT-2-small-shaped leg:", json.dumps(gpt2))
    ceiling = None if (args.skip_clock or profiled) else bench_mfma_ceiling(tw, si, torch)
    log("[bench] matrix-instruction ceiling:", json.dumps(ceiling))
    ablation = None if args.skip_ablation else bench_latency_ablation(args, tw, si, torch)
    if ablation:
        log("[bench] latency ablation (GPT-2-small shape):", json.dumps(ablation))
    cpu = None if args.skip_cpu else cpu_baseline(si)

    g = train["gemm"]
    out = {
        "metric": "subnet train tokens/s (fwd+bwd, %MFMA peak) + extract/aggregate GB/s (%HBM peak)",
        "value": train["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": train["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "llama1b_round: configs[2], 22 layers d=2048 16x128 heads SwiGLU 5632 vocab 32000, S=4 overlapping half-width "
                               f"subnets, batch 4x2048 Zipf(1.1) tokens, {args.local_steps} local AdamW steps per subnet, sample+extract+train+aggregate; "
                               "output projections stored unit-major",
                   "S": 4, "batch": 4, "seq_len": 2048, "local_steps": args.local_steps},
        "roofline": {"bound": "mfma", "kernel": "gemm_pp_kernel / gemm_mfma_kernel: every projection launch of one forward+backward per subnet, "
                                                 "kernels serialised on one stream",
                     "achieved": g["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": g["tflops"] / PEAK_BF16_TFLOPS,
                     "traffic": TRAFFIC_PROJECTION_LAUNCH, "traffic_unit": "bytes per launch behind the L2 (rocprofv3 FETCH_SIZE/WRITE_SIZE, calibrated)",
                     "algorithmic_bytes_per_launch": g["algorithmic_bytes_per_launch"],
                     "avg_launch_ms": g["avg_ms"], "launches": g["launches"], "flops_per_launch": g["flops_per_launch"]},
        "fwd_bwd": {"tokens_per_s": train["fwd_bwd_tokens_per_s"], "ms": train["fwd_bwd_ms"], "median_ms": train["fwd_bwd_median_ms"],
                    "min_ms": train["fwd_bwd_min_ms"], "timed_calls": train["fwd_bwd_timed_calls"], "tflops": train["fwd_bwd_tflops"],
                    "frac_mfma_peak": train["fwd_bwd_frac_mfma_peak"]},
        "phase_ms_per_step": train["phase_ms_per_step"],
        **({"native_round": train["native_round"]} if "native_round" in train else {}),
        "cpu_baseline": cpu,
    }
    if movers:
        out["movers_llama7b_stack"] = movers
        out["roofline_movers"] = {
            "bound": "hbm", "kernel": "extract_kernel / aggregate_rows_kernel at configs[3] (32 layers d=4096, S=8, 50%), output projections unit-major",
            "achieved": (movers["extract_alg_GB"] + movers["aggregate_alg_GB"]) / ((movers["extract_ms"] + movers["aggregate_ms"]) * 1e-3),
            "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": (movers["extract_alg_GB"] + movers["aggregate_alg_GB"]) / ((movers["extract_ms"] + movers["aggregate_ms"]) * 1e-3) / PEAK_HBM_GBS,
            "traffic": 8 * TRAFFIC_EXTRACT_LAYER_LAUNCH + TRAFFIC_AGGREGATE_LAYER_LAUNCH,
            "traffic_unit": "bytes per layer (its share of the 8 per-subnet extracts and of the aggregate; a launch carries 4 layers) behind the L2",
            "algorithmic_bytes_per_layer": (movers["extract_alg_GB"] + movers["aggregate_alg_GB"]) * 1e9 / 32,
            # twist_extract_all reads each central element once for all 8 subnets: the bytes it moves are FEWER than the
            # per-subnet algorithmic count above, so its rate is quoted on what it moves (and, for comparison, on that count)
            "with_one_pass_extract": {
                "extract_all_ms": movers["extract_all_ms"], "moved_GB": movers["extract_all_moved_GB"] + movers["aggregate_alg_GB"],
                "achieved_on_moved_bytes": (movers["extract_all_moved_GB"] + movers["aggregate_alg_GB"]) / ((movers["extract_all_ms"] + movers["aggregate_ms"]) * 1e-3),
                "achieved_on_per_subnet_bytes": (movers["extract_alg_GB"] + movers["aggregate_alg_GB"]) / ((movers["extract_all_ms"] + movers["aggregate_ms"]) * 1e-3)}}
        out["movers_llama7b_stack_out_in_layout"] = movers_rm
    if not args.skip_cpu and not args.skip_movers:
        out["cpu_baseline_movers"] = cpu_baseline_movers(si)
        log("[bench] cpu baseline (movers):", json.dumps(out["cpu_baseline_movers"]))
    if clock:
        out["clock_under_projection_load"] = clock
    if golden:
        out["golden_ticket_llama7b_fwd_bwd"] = golden
    if gpt2:
        out["gpt2_small_4_subnets"] = gpt2
    if ceiling:
        out["mfma_only_ceiling"] = ceiling
    if cpu and not args.skip_cpu:
        try:
            out["cpu_baseline_one_thread"] = cpu_baseline_one_thread(si)
            log("[bench] cpu baseline (one thread):", json.dumps(out["cpu_baseline_one_thread"]))
        except ImportError:
            pass
    if ablation:
        out["latency_ablation_gpt2_small"] = ablation
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
