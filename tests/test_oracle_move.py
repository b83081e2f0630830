"""Pins for the checker's dispatcher (extract) and aggregator (Sections 3.2, 3.3, Appendix C)."""
import os
from dataclasses import replace

import numpy as np
import pytest

import synth_inputs as si
from oracle import move
from oracle.sample import KIND_FFN, KIND_HEAD, sample_plan

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _count(P):
    return sum(v.size for lw in P["layers"] for v in lw.values()) + sum(v.size for v in P["globals"].values())


def test_table2_communication_column():
    """Traffic is proportional to the parameters a subnet holds (Appendix C).  With GPT-2 124M,
    12 blocks per module and the first/last two layers shared, 45.50 TB x N_model(kappa) / N_model(full)
    must reproduce every entry of Table 2's communication column."""
    cfg = replace(si.CFG2, ffn_granule=3072 // 12)
    full = {"layers": [{k: np.zeros(s, np.int8) for k, s in si.layer_shapes(cfg).items()} for _ in range(12)],
            "globals": {k: np.zeros(s, np.int8) for k, s in si.global_shapes(cfg).items()}}
    n_full = _count(full)
    assert n_full == 124_439_808                     # GPT-2 small
    # Appendix C closed forms for one full layer
    d, da, df = 768, 768, 3072
    n_attn = 4 * da * d + 3 * da + d
    n_ffn = 2 * df * d + df + d
    assert sum(v.size for v in full["layers"][0].values()) == n_attn + n_ffn + 2 * (2 * d)
    shared = [1, 1] + [0] * 8 + [1, 1]
    rows = [l.split() for l in open(os.path.join(GOLD, "table2_comm_tb.txt")) if not l.startswith("#")]
    ddp = [float(v) for s, k, v in rows if s == "ddp"][0]
    for setting, k, want in rows:
        if setting == "ddp":
            continue
        k = int(k)
        hs = k if setting in ("attn", "both") else 12
        fs = k if setting in ("ffn", "both") else 12
        plan = sample_plan(12, 12, 12, 4, hs, fs, seed=1, layer_shared=shared)
        sub = move.extract(full, plan, 0, cfg.d_head, cfg.ffn_granule)
        n_sub = _count(sub)
        # closed form of Appendix C with the exact per-tensor counts
        part_attn = 4 * da * d + 3 * da
        part_ffn = 2 * df * d + df
        assert n_sub == n_full - 8 * (part_attn * (12 - hs) // 12 + part_ffn * (12 - fs) // 12)
        assert abs(ddp * n_sub / n_full - float(want)) <= 0.0101, (setting, k, ddp * n_sub / n_full, want)


def _tiny(seed=0, arch="gpt"):
    if arch == "gpt":
        cfg = si.ModelCfg(n_layers=2, d_model=8, n_heads=4, d_head=2, d_ff=12, ffn_granule=3, vocab=11, max_seq=8)
    else:
        cfg = si.ModelCfg(arch="llama", n_layers=2, d_model=8, n_heads=4, d_head=2, d_ff=12, ffn_granule=1, vocab=11,
                          max_seq=8, act="swiglu", norm="rms", has_bias=False, tied_head=False, rope=True)
    return cfg, si.make_weights(cfg, seed, std=0.5, generic=True)


def test_extract_picks_the_right_blocks_by_hand():
    cfg, full = _tiny()
    plan = sample_plan(2, 4, 4, 2, 2, 2, seed=3)
    for s in range(2):
        sub = move.extract(full, plan, s, cfg.d_head, cfg.ffn_granule)
        for l in range(2):
            heads = plan[l][KIND_HEAD]["idx"][s]
            units = plan[l][KIND_FFN]["idx"][s]
            lw, sw = full["layers"][l], sub["layers"][l]
            for k, h in enumerate(heads):                 # head h = d_head rows of W^Q.. and columns of C^attn
                for name in ("wq", "wk", "wv", "bq", "bk", "bv"):
                    assert np.array_equal(sw[name][k * 2:(k + 1) * 2], lw[name][h * 2:(h + 1) * 2])
                assert np.array_equal(sw["wo"][:, k * 2:(k + 1) * 2], lw["wo"][:, h * 2:(h + 1) * 2])
            for k, u in enumerate(units):                 # FFN block u = granule rows of W^ffn, columns of C^ffn
                assert np.array_equal(sw["w_up"][k * 3:(k + 1) * 3], lw["w_up"][u * 3:(u + 1) * 3])
                assert np.array_equal(sw["b_up"][k * 3:(k + 1) * 3], lw["b_up"][u * 3:(u + 1) * 3])
                assert np.array_equal(sw["w_down"][:, k * 3:(k + 1) * 3], lw["w_down"][:, u * 3:(u + 1) * 3])
            for name in ("bo", "b_down", "norm1_w", "norm1_b", "norm2_w", "norm2_b"):
                assert np.array_equal(sw[name], lw[name])
            assert sw["wq"].shape == (4, 8) and sw["wo"].shape == (8, 4) and sw["w_down"].shape == (8, 6)
        assert all(np.array_equal(sub["globals"][k], full["globals"][k]) for k in full["globals"])


def _perturbed(cfg, full, plan, S, seed=9):
    subs = []
    for s in range(S):
        sub = move.extract(full, plan, s, cfg.d_head, cfg.ffn_granule)
        for l, lw in enumerate(sub["layers"]):
            for k in lw:
                lw[k] = lw[k] + si.perturbation(seed, f"{s}.{l}.{k}", lw[k].shape, 0.1)
        for k in sub["globals"]:
            sub["globals"][k] = sub["globals"][k] + si.perturbation(seed, f"{s}.g.{k}", sub["globals"][k].shape, 0.1)
        subs.append(sub)
    return subs


@pytest.mark.parametrize("arch", ["gpt", "llama"])
def test_aggregate_matches_formula_by_brute_force(arch):
    """p = sum_i p_i 1[p in W_i] / sum_i 1[p in W_i], one scalar at a time in pure Python."""
    cfg, full = _tiny(1, arch)
    S = 3
    plan = sample_plan(2, 4, cfg.n_ffn_units, S, 2, cfg.n_ffn_units // 2, seed=4)
    subs = _perturbed(cfg, full, plan, S)
    new = move.aggregate(full, plan, subs, cfg.d_head, cfg.ffn_granule)
    for l, lw in enumerate(full["layers"]):
        for name, w in lw.items():
            if name not in move.PARTITIONED:
                assert np.allclose(new["layers"][l][name], sum(s_["layers"][l][name] for s_ in subs) / S, rtol=1e-14)
                continue
            kind, axis = move.PARTITIONED[name]
            qb = cfg.d_head if kind == KIND_HEAD else cfg.ffn_granule
            it = np.ndindex(*w.shape)
            for pos in it:
                e = pos[axis]
                u, r = divmod(e, qb)
                num, den = 0.0, 0
                for s in range(S):
                    row = plan[l][kind]["idx"][s]
                    if u in row:
                        k = row.index(u)
                        sp = list(pos)
                        sp[axis] = k * qb + r
                        num += subs[s]["layers"][l][name][tuple(sp)]
                        den += 1
                want = num / den if den else w[pos]
                assert abs(new["layers"][l][name][pos] - want) < 1e-14
    for name in full["globals"]:
        assert np.allclose(new["globals"][name], sum(s_["globals"][name] for s_ in subs) / S, rtol=1e-14)


def test_partition_roundtrip_is_identity():
    """Disjoint subnets that were not trained aggregate back to the central model exactly."""
    cfg, full = _tiny(2)
    plan = sample_plan(2, 4, 4, 2, 2, 2, seed=0)      # tight bound -> exact partition
    subs = [move.extract(full, plan, s, cfg.d_head, cfg.ffn_granule) for s in range(2)]
    new = move.aggregate(full, plan, subs, cfg.d_head, cfg.ffn_granule)
    for l in range(2):
        for k in full["layers"][l]:
            assert np.array_equal(new["layers"][l][k], full["layers"][l][k]), k
    # and a trained partition aggregates to the concatenation: each unit takes its only owner's value
    subs = _perturbed(cfg, full, plan, 2)
    new = move.aggregate(full, plan, subs, cfg.d_head, cfg.ffn_granule)
    for s in range(2):
        back = move.extract(new, plan, s, cfg.d_head, cfg.ffn_granule)
        for name in move.PARTITIONED:
            if name in back["layers"][0]:
                assert np.array_equal(back["layers"][1][name], subs[s]["layers"][1][name])


def test_full_width_subnets_average_to_plain_mean():
    cfg, full = _tiny(3)
    S = 3
    plan = sample_plan(2, 4, 4, S, 4, 4, seed=0)      # N_sub = N_full
    subs = _perturbed(cfg, full, plan, S)
    new = move.aggregate(full, plan, subs, cfg.d_head, cfg.ffn_granule)
    for l in range(2):
        for k in full["layers"][l]:
            assert np.allclose(new["layers"][l][k], sum(s_["layers"][l][k] for s_ in subs) / S, rtol=1e-14, atol=0)
    same = [move.extract(full, plan, s, cfg.d_head, cfg.ffn_granule) for s in range(S)]
    new = move.aggregate(full, plan, same, cfg.d_head, cfg.ffn_granule)
    for l in range(2):
        for k in full["layers"][l]:
            assert np.allclose(new["layers"][l][k], full["layers"][l][k], rtol=1e-15, atol=0)


def test_missing_subnet_leaves_its_exclusive_units_unchanged():
    cfg, full = _tiny(4)
    plan = sample_plan(2, 4, 4, 2, 2, 2, seed=0)      # partition: every unit has exactly one owner
    subs = _perturbed(cfg, full, plan, 2)
    new = move.aggregate(full, plan, {0: subs[0]}, cfg.d_head, cfg.ffn_granule)
    kept = move.extract(new, plan, 1, cfg.d_head, cfg.ffn_granule)
    orig = move.extract(full, plan, 1, cfg.d_head, cfg.ffn_granule)
    took = move.extract(new, plan, 0, cfg.d_head, cfg.ffn_granule)
    for name in ("wq", "wo", "w_up", "w_down", "bq", "b_up"):
        assert np.array_equal(kept["layers"][0][name], orig["layers"][0][name])
        assert np.array_equal(took["layers"][0][name], subs[0]["layers"][0][name])
