"""Train-at-X / evaluate-at-Y harness (Section 5.1, "Architectural Robustness": a model trained with subnets of X
blocks is evaluated, without retraining, through deployment subnets of Y blocks).

Loops and bookkeeping only: sampling, extraction, training steps, aggregation and evaluation are the library's
entry points (twist_round, twist_sample in deployment mode, twist_extract, twist_subnet_forward).  Perplexity on
the paper's data set needs that data set and trained weights; on synthetic weights the grid's entries are evaluation
losses, which is what the checker can reproduce.
"""
from __future__ import annotations

import torch

from . import binding as tw


def robustness_grid(ctx: "tw.Context", layers, globs, train_batches, eval_batch, blocks_total: int, xs, ys, *, S: int, rounds: int,
                    opt: dict, seed: int = 0, layer_shared=None, eval_seed: int = 1000):
    """grid[X][Y] = evaluation loss of a deployment subnet keeping Y of `blocks_total` heads and FFN blocks per layer, cut
    from the central model after `rounds` TwIST rounds with S subnets of X blocks each.

    layers / globs: the central model's tensors (dicts of CUDA tensors as for FullWeights); they are restored after
    every X.  train_batches(x_blocks, r) -> (inputs, targets) of shape [S, local_steps, B, N(, d)] for round r;
    eval_batch = (inputs, targets) of shape [B, N(, d)].  Every block kind keeps the same number of blocks, as in the
    paper's "both" setting.  X = blocks_total trains the full model (one full-width "subnet" per worker, plain
    averaging)."""
    start = ([{k: v.clone() for k, v in lw.items()} for lw in layers], {k: v.clone() for k, v in globs.items()})
    fw = tw.FullWeights(layers, globs)
    ex, ey = eval_batch
    B, N = ex.shape[0], ex.shape[1]
    grid = {}
    for X in xs:
        for lw, l0 in zip(layers, start[0]):
            for k in lw:
                lw[k].copy_(l0[k])
        for k in globs:
            globs[k].copy_(start[1][k])
        for r in range(rounds):
            x, y = train_batches(X, r)
            steps = x.shape[1]
            sb, wb, ib = ctx.twist_round_bytes(S, X, X, x.shape[2], x.shape[3], steps, opt=opt, layer_shared=layer_shared)
            slab, ws, image = (torch.empty(n, dtype=torch.uint8, device="cuda") for n in (sb, wb, ib))
            losses = torch.zeros(S, steps, device="cuda")
            ctx.twist_round(fw, x, y, S, X, X, slab, ws, image, losses, seed=seed, rnd=r, opt=opt, layer_shared=layer_shared)
        row = {}
        for Y in ys:
            plan = ctx.twist_sample(1, Y, Y, seed=eval_seed, require_coverage=False, layer_shared=layer_shared)
            sub = ctx.twist_extract(plan, fw, 0)
            ws = torch.empty(ctx.twist_workspace_bytes(sub, B, N), dtype=torch.uint8, device="cuda")
            loss = torch.zeros(1, device="cuda")
            ctx.twist_subnet_forward(sub, ex, ey, ws, loss)
            row[Y] = loss.item()
            sub.close()
            plan.close()
        grid[X] = row
    for lw, l0 in zip(layers, start[0]):
        for k in lw:
            lw[k].copy_(l0[k])
    for k in globs:
        globs[k].copy_(start[1][k])
    return grid
