"""GPU parity of twist_sample / twist_extract / twist_aggregate against the CPU checker, through the C ABI."""
import os
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as si
from helpers import _stored, bf16_ulp_distance, model_to_numpy, rel_fro, subnet_to_numpy, to_device, to_numpy
from oracle import move as omove
from oracle.sample import sample_plan

pytestmark = pytest.mark.gpu


def _ctx(lib, cfg):
    return lib.Context(lib.desc_from_cfg(cfg))


# ------------------------------------------------------------------------------------------ sample
SAMPLE_CASES = [
    # (n_layers, heads, d_head, d_ff, granule, S, heads_sub, ffn_sub, common_heads, common_ffn, shared, coverage)
    (2, 4, 32, 512, 1, 2, 2, 256, (), (), None, True),                    # workload 1: tight bound, partition
    (3, 12, 64, 3072, 1, 4, 3, 768, (), (), None, True),                  # workload 2
    (2, 16, 128, 5632, 1, 4, 8, 2816, (), (), None, True),                # workload 3: overlap, covered
    (2, 32, 128, 11008, 1, 8, 16, 5504, (), (), None, True),              # workload 4
    (4, 12, 64, 3072, 256, 4, 6, 8, (0, 5), (3,), [1, 0, 0, 1], True),    # blocks of 256 neurons, common sets, shared layers
    (2, 32, 128, 11008, 1, 1, 16, 5504, (), (), None, False),             # deployment: one subnet, no coverage
    (2, 7, 32, 33, 3, 3, 5, 6, (2,), (), None, True),                     # odd sizes
    (13, 16, 128, 5632, 1, 4, 8, 2816, (1,), (7, 4000), None, True),      # 26 tables: more than the library's host threads
]


@pytest.mark.parametrize("case", SAMPLE_CASES)
def test_sample_matches_oracle_bit_exactly(lib, case):
    L, H, dh, F, g, S, hs, fs, ch, cf, shared, cov = case
    cfg = si.ModelCfg(n_layers=L, d_model=64, n_heads=H, d_head=dh, d_ff=F, ffn_granule=g)
    ctx = _ctx(lib, cfg)
    for seed, rnd in ((0, 0), (12345, 7)):
        plan = ctx.twist_sample(S, hs, fs, seed=seed, rnd=rnd, common_heads=ch, common_ffn=cf, layer_shared=shared, require_coverage=cov)
        want = sample_plan(L, H, F // g, S, hs, fs, seed, rnd, ch, cf, shared, cov)
        for l in range(L):
            for kind in (0, 1):
                idx, inv, cnt = plan.twist_plan_view(l, kind)
                w = want[l][kind]
                assert idx.tolist() == w["idx"], (l, kind)
                assert inv.tolist() == w["inv"]
                assert cnt.tolist() == w["count"]
                # the device copies, read back, hold the same integers
                d_idx, d_inv, d_cnt = plan.twist_plan_read_device(l, kind)
                assert d_idx.tolist() == w["idx"] and d_inv.tolist() == w["inv"] and d_cnt.tolist() == w["count"], (l, kind)
                assert plan.device_tables(l, kind)[3:] == (w["n_sub"], w["n_full"])
        plan.close()


def test_sample_matches_oracle_on_a_seeded_sweep_of_settings(lib):
    """Sixty seeded settings of Algorithm 1 (sizes, subnet counts, common sets, coverage on and off, shared layers),
    every table bit for bit against the checker."""
    rng = np.random.default_rng(2024)
    done = 0
    while done < 60:
        H, U = int(rng.integers(1, 20)), int(rng.integers(1, 70))
        S = int(rng.integers(1, 9))
        hs, fs = int(rng.integers(1, H + 1)), int(rng.integers(1, U + 1))
        ch = tuple(sorted(rng.choice(H, size=int(rng.integers(0, min(hs, 3) + 1)), replace=False).tolist()))
        cf = tuple(sorted(rng.choice(U, size=int(rng.integers(0, min(fs, 4) + 1)), replace=False).tolist()))
        cov = bool(rng.integers(0, 2))
        if cov and (H - len(ch) > S * (hs - len(ch)) or U - len(cf) > S * (fs - len(cf))):
            continue                                  # violates the size bound below Algorithm 1: covered elsewhere
        L = int(rng.integers(1, 4))
        shared = [int(x) for x in rng.integers(0, 2, size=L)] if rng.integers(0, 2) else None
        seed, rnd = int(rng.integers(0, 2**31)), int(rng.integers(0, 50))
        cfg = si.ModelCfg(n_layers=L, d_model=16, n_heads=H, d_head=8, d_ff=U * 2, ffn_granule=2, vocab=0)
        ctx = _ctx(lib, cfg)
        plan = ctx.twist_sample(S, hs, fs, seed=seed, rnd=rnd, common_heads=ch, common_ffn=cf, layer_shared=shared, require_coverage=cov)
        want = sample_plan(L, H, U, S, hs, fs, seed, rnd, ch, cf, shared, cov)
        for l in range(L):
            for kind in (0, 1):
                idx, inv, cnt = plan.twist_plan_view(l, kind)
                w = want[l][kind]
                assert idx.tolist() == w["idx"] and inv.tolist() == w["inv"] and cnt.tolist() == w["count"], (done, l, kind, H, U, S, hs, fs, ch, cf, cov)
        plan.close()
        ctx.close()
        done += 1


def test_sample_rejects_bound_violations(lib):
    ctx = _ctx(lib, si.CFG1)
    with pytest.raises(lib.TwistError) as e:
        ctx.twist_sample(2, 1, 256)
    assert e.value.status == 2
    with pytest.raises(lib.TwistError):
        ctx.twist_sample(2, 2, 255)
    with pytest.raises(lib.TwistError):
        ctx.twist_sample(2, 2, 513)
    ctx.twist_sample(1, 1, 17, require_coverage=False).close()      # deployment relaxes the coverage bound


# ------------------------------------------------------------------------------------------ extract / aggregate
SMALL = {
    "cfg1_f32": (si.CFG1, 2, 2, 256),
    "gpt_bf16": (replace(si.CFG2, n_layers=2, vocab=1000, max_seq=64), 4, 3, 768),
    "llama_bf16": (replace(si.CFG3, n_layers=2, d_model=512, n_heads=8, d_head=64, d_ff=1408, vocab=777, max_seq=64), 4, 4, 704),
    "llama_overlap_S8": (replace(si.CFG4, n_layers=2, d_model=256, n_heads=8, d_head=32, d_ff=1000), 8, 4, 500),
    "gpt_blocks_f32": (replace(si.CFG1, n_layers=3, d_ff=768, ffn_granule=64, vocab=50, max_seq=16), 3, 2, 5),
    "ragged_f32": (si.ModelCfg(n_layers=2, d_model=36, n_heads=5, d_head=6, d_ff=70, ffn_granule=7, vocab=19, max_seq=8), 3, 2, 4),
    "ragged_bf16": (si.ModelCfg(n_layers=1, d_model=100, n_heads=3, d_head=10, d_ff=99, ffn_granule=1, vocab=0, dtype="bf16"), 2, 2, 60),
}
# nearly every neuron kept and rows of odd length: the spans of the down projection's element path are as long as a
# tile allows and start at a different misalignment in every row
SMALL["wide_odd_bf16"] = (si.ModelCfg(n_layers=1, d_model=40, n_heads=2, d_head=8, d_ff=1101, ffn_granule=1, vocab=0, dtype="bf16"), 2, 1, 1100)
SMALL["wide_odd_f32"] = (si.ModelCfg(n_layers=1, d_model=24, n_heads=2, d_head=8, d_ff=1101, ffn_granule=1, vocab=0), 3, 2, 1101)
# more layers than one launch's job table holds (two such layers fit): the movers cut the model into several launches
SMALL["gpt_12layers_f32"] = (replace(si.CFG1, n_layers=12, d_model=32, n_heads=4, d_head=8, d_ff=96, vocab=40, max_seq=8), 3, 2, 40)
SMALL["llama_11layers_bf16"] = (replace(si.CFG3, n_layers=11, d_model=64, n_heads=4, d_head=16, d_ff=136, vocab=50, max_seq=8), 4, 2, 70)
# nine subnets: one more than the one-pass kernels handle at once (twist_extract_all falls back to per-subnet gathers,
# twist_aggregate to its chunked general kernel)
SMALL["gpt_S9_bf16"] = (replace(si.CFG2, n_layers=1, d_model=256, n_heads=12, d_head=64, d_ff=1024, vocab=300, max_seq=32), 9, 2, 128)
# the same shapes with the output projections stored unit-major (every partitioned tensor cut along rows)
for _k in ("cfg1_f32", "gpt_bf16", "llama_bf16", "llama_overlap_S8", "ragged_f32", "ragged_bf16"):
    SMALL[_k + "_um"] = (replace(SMALL[_k][0], out_unit_major=True),) + SMALL[_k][1:]


def _setup(lib, name, seed=0, **kw):
    cfg, S, hs, fs = SMALL[name]
    full_np = si.make_weights(cfg, seed, generic=True)
    full_t = to_device(full_np, cfg)
    ctx = _ctx(lib, cfg)
    plan = ctx.twist_sample(S, hs, fs, seed=seed + 1, **kw)
    oplan = sample_plan(cfg.n_layers, cfg.n_heads, cfg.n_ffn_units, S, hs, fs, seed + 1,
                        layer_shared=kw.get("layer_shared"), require_coverage=kw.get("require_coverage", True))
    fw = lib.FullWeights(full_t["layers"], full_t["globals"])
    return cfg, S, full_np, full_t, ctx, plan, oplan, fw


@pytest.mark.parametrize("name", list(SMALL))
def test_extract_is_a_bit_exact_gather(lib, name):
    cfg, S, full_np, full_t, ctx, plan, oplan, fw = _setup(lib, name)
    for s in range(S):
        sub = ctx.twist_extract(plan, fw, s)
        got = subnet_to_numpy(sub, cfg)
        want = omove.extract(full_np, oplan, s, cfg.d_head, cfg.ffn_granule)
        for l in range(cfg.n_layers):
            for k, w in want["layers"][l].items():
                assert got["layers"][l][k].shape == w.shape, (l, k)
                assert np.array_equal(got["layers"][l][k], w), (name, s, l, k)
        for k, w in want["globals"].items():
            assert np.array_equal(got["globals"][k], w), k
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", list(SMALL))
def test_extract_all_equals_the_per_subnet_extract_bit_for_bit(lib, name):
    """twist_extract_all (one pass over the central model for all subnets) against twist_extract, whole slabs compared."""
    cfg, S, full_np, full_t, ctx, plan, oplan, fw = _setup(lib, name, seed=12)
    for store in (lib.STORE_PARAMS, lib.STORE_GRADS):
        nb = ctx.twist_subnet_bytes(plan, store)
        marks = [torch.full((nb,), 0x5A, dtype=torch.uint8, device="cuda") for _ in range(S)]   # same filler in both, so padding compares too
        both = ctx.twist_extract_all(plan, fw, store=store, storages=marks)
        for s in range(S):
            one = ctx.twist_extract(plan, fw, s, store=store, storage=torch.full((nb,), 0x5A, dtype=torch.uint8, device="cuda"))
            assert torch.equal(one.storage, both[s].storage), (name, store, s)
    want = omove.extract(full_np, oplan, S - 1, cfg.d_head, cfg.ffn_granule)      # and against the checker directly
    got = subnet_to_numpy(both[S - 1], cfg)
    for l in range(cfg.n_layers):
        for k, w in want["layers"][l].items():
            assert np.array_equal(got["layers"][l][k], w), (name, l, k)


def _perturb(cfg, sub, s, seed=5):
    """Stand-in for local training: add N(0, 1e-3) noise to every subnet tensor, same on both sides."""
    pert = {}
    for l in range(cfg.n_layers):
        for k in si.layer_shapes(cfg):
            v = sub.twist_subnet_view(l, k)
            n = si.perturbation(seed, f"{s}.{l}.{k}", tuple(_stored(cfg, k, v).shape))     # drawn in [out, in]
            v.add_(torch.tensor(np.ascontiguousarray(_stored(cfg, k, n)), dtype=torch.float64).to(v.dtype).cuda())
    for k in si.global_shapes(cfg):
        v = sub.twist_subnet_view(-1, k)
        v.add_(torch.tensor(si.perturbation(seed, f"{s}.g.{k}", tuple(v.shape)), dtype=torch.float64).to(v.dtype).cuda())


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("drop", [False, True])
def test_aggregate_matches_formula(lib, name, drop):
    cfg, S, full_np, full_t, ctx, plan, oplan, fw = _setup(lib, name, seed=3)
    subs = [ctx.twist_extract(plan, fw, s) for s in range(S)]
    for s, sub in enumerate(subs):
        _perturb(cfg, sub, s)
    use = list(range(S))
    if drop:
        use = use[1:] if S > 1 else use      # a worker that never reports back
        use = use[::-1]                       # and an arbitrary order
    sub_np = {s: subnet_to_numpy(subs[s], cfg) for s in use}
    want = omove.aggregate(full_np, oplan, sub_np, cfg.d_head, cfg.ffn_granule)
    ctx.twist_aggregate(plan, [subs[s] for s in use], fw)
    got = model_to_numpy(full_t, cfg)
    tol = 5e-3 if cfg.dtype == "bf16" else 1e-4
    for l in range(cfg.n_layers):
        for k, w in want["layers"][l].items():
            g = got["layers"][l][k]
            assert rel_fro(g, w) <= tol, (name, l, k, rel_fro(g, w))
            if cfg.dtype == "bf16":
                assert bf16_ulp_distance(g, si.to_bf16_grid(w)).max() <= 1, (l, k)
            else:
                np.testing.assert_allclose(g, w, rtol=3e-7, atol=1e-9)
            # single-owner and ownerless parameters are exact copies
            if k in omove.PARTITIONED:
                kind, axis = omove.PARTITIONED[k]
                q = cfg.d_head if kind == 0 else cfg.ffn_granule
                cnt = np.zeros(oplan[l][kind]["n_full"], int)
                for s in use:
                    cnt[oplan[l][kind]["idx"][s]] += 1
                e = np.repeat(cnt, q)
                sel = e <= 1
                gs, ws = (g[sel], w[sel]) if axis == 0 else (g[:, sel], w[:, sel])
                assert np.array_equal(gs, ws), (l, k)
    for k, w in want["globals"].items():
        assert rel_fro(got["globals"][k], w) <= tol


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("drop", [False, True])
def test_running_sum_aggregate_equals_the_one_shot_aggregate_bit_for_bit(lib, name, drop):
    """twist_aggregate_begin/add/finish with one subnet resident at a time, against twist_aggregate over all of them."""
    cfg, S, full_np, full_t, ctx, plan, oplan, fw = _setup(lib, name, seed=11)
    other_t = to_device(full_np, cfg)
    fw2 = lib.FullWeights(other_t["layers"], other_t["globals"])
    subs = [ctx.twist_extract(plan, fw, s) for s in range(S)]
    for s, sub in enumerate(subs):
        _perturb(cfg, sub, s)
    use = list(range(S))
    if drop:
        use = (use[1:] if S > 1 else use)[::-1]
    ctx.twist_aggregate(plan, [subs[s] for s in use], fw)
    image = torch.full((ctx.twist_aggregate_image_bytes() // 4,), float("nan"), device="cuda").view(torch.uint8)   # need not be cleared
    acc = ctx.twist_aggregate_begin(plan, image)
    slab = torch.empty(ctx.twist_subnet_bytes(plan), dtype=torch.uint8, device="cuda")      # ONE subnet's storage, reused
    for s in use:
        one = ctx.twist_extract(plan, fw2, s, storage=slab)      # re-create subnet s in the shared slab ...
        slab.copy_(subs[s].storage)                               # ... with its trained values
        acc.twist_aggregate_add(one)
        with pytest.raises(lib.TwistError):
            acc.twist_aggregate_add(one)                          # a blueprint row reports once
    acc.twist_aggregate_finish(fw2)
    for l in range(cfg.n_layers):
        for k in full_t["layers"][l]:
            assert torch.equal(full_t["layers"][l][k].view(torch.uint8), other_t["layers"][l][k].view(torch.uint8)), (name, l, k)
    for k in full_t["globals"]:
        assert torch.equal(full_t["globals"][k].view(torch.uint8), other_t["globals"][k].view(torch.uint8)), (name, k)
    # independent of the one-shot kernel: the formula itself, on the tensors of the last layer
    sub_np = {s: subnet_to_numpy(subs[s], cfg) for s in use}
    want = omove.aggregate(full_np, oplan, sub_np, cfg.d_head, cfg.ffn_granule)
    got = model_to_numpy(other_t, cfg)
    tol = 5e-3 if cfg.dtype == "bf16" else 1e-4
    for k, w in want["layers"][-1].items():
        assert rel_fro(got["layers"][-1][k], w) <= tol, (name, k)
    # finish forgot the added rows: the same object serves another pass, and nothing added leaves the model alone
    before = {k: v.clone() for k, v in other_t["layers"][0].items()}
    acc.twist_aggregate_finish(fw2)
    for k, v in before.items():
        assert torch.equal(v.view(torch.uint8), other_t["layers"][0][k].view(torch.uint8)), k
    acc.close()


def test_movers_on_a_seeded_sweep_of_ragged_shapes(lib):
    """Twenty-four seeded small models with awkward sizes (odd widths, granules, subnet counts up to 9, both dtypes, both
    layouts; every fourth one with a wide FFN cut into single neurons): extract and extract_all bit for bit against the checker, aggregate within tolerance, and the running-sum
    aggregate bit for bit against the one-shot aggregate."""
    rng = np.random.default_rng(int(os.environ.get("TWIST_SWEEP_SEED", "77")))      # other seeds / more cases for a longer soak
    for case in range(int(os.environ.get("TWIST_SWEEP_CASES", "24"))):
        H, dh = int(rng.integers(1, 8)), int(rng.choice([2, 6, 8, 10, 16, 24, 32]))
        g = int(rng.choice([1, 1, 2, 3, 8]))
        U = int(rng.integers(2, 40))
        if case % 4 == 3:        # wide FFN with single-neuron blocks: the element path's spans reach a full tile
            g, U = 1, int(rng.integers(300, 1300))
        S = int(rng.integers(1, 10))
        hs, fs = int(rng.integers(max(1, -(-H // S)), H + 1)), int(rng.integers(max(1, -(-U // S)), U + 1))
        cfg = si.ModelCfg(n_layers=int(rng.integers(1, 3)), d_model=int(rng.choice([8, 12, 36, 64, 100, 256])), n_heads=H, d_head=dh, d_ff=U * g,
                          ffn_granule=g, vocab=int(rng.choice([0, 37])), max_seq=8, dtype=str(rng.choice(["f32", "bf16"])),
                          out_unit_major=bool(rng.integers(0, 2)))
        tag = (case, H, dh, g, U, S, hs, fs, cfg.d_model, cfg.dtype, cfg.out_unit_major, cfg.vocab)
        full_np = si.make_weights(cfg, 100 + case, generic=True)
        full_t, other_t = to_device(full_np, cfg), to_device(full_np, cfg)
        ctx = _ctx(lib, cfg)
        plan = ctx.twist_sample(S, hs, fs, seed=case)
        oplan = sample_plan(cfg.n_layers, H, U, S, hs, fs, case)
        fw, fw2 = lib.FullWeights(full_t["layers"], full_t["globals"]), lib.FullWeights(other_t["layers"], other_t["globals"])
        subs = ctx.twist_extract_all(plan, fw)
        for s in range(S):
            want = omove.extract(full_np, oplan, s, dh, g)
            got = subnet_to_numpy(subs[s], cfg)
            one = subnet_to_numpy(ctx.twist_extract(plan, fw, s), cfg)
            for l in range(cfg.n_layers):
                for k, w in want["layers"][l].items():
                    assert np.array_equal(got["layers"][l][k], w) and np.array_equal(one["layers"][l][k], w), (tag, s, l, k)
            for k, w in want["globals"].items():
                assert np.array_equal(got["globals"][k], w), (tag, s, k)
        for s, sub in enumerate(subs):
            _perturb(cfg, sub, s, seed=case)
        use = list(range(S))[::-1] if case % 3 == 0 else list(range(S))
        if case % 4 == 1 and S > 1:
            use = use[1:]
        want = omove.aggregate(full_np, oplan, {s: subnet_to_numpy(subs[s], cfg) for s in use}, dh, g)
        ctx.twist_aggregate(plan, [subs[s] for s in use], fw)
        acc = ctx.twist_aggregate_begin(plan)
        for s in use:
            acc.twist_aggregate_add(subs[s])
        acc.twist_aggregate_finish(fw2)
        got = model_to_numpy(full_t, cfg)
        tol = 5e-3 if cfg.dtype == "bf16" else 1e-4
        for l in range(cfg.n_layers):
            for k, w in want["layers"][l].items():
                assert rel_fro(got["layers"][l][k], w) <= tol, (tag, l, k)
                assert torch.equal(full_t["layers"][l][k].view(torch.uint8), other_t["layers"][l][k].view(torch.uint8)), (tag, l, k)
        for k, w in want["globals"].items():
            assert rel_fro(got["globals"][k], w) <= tol, (tag, k)
            assert torch.equal(full_t["globals"][k].view(torch.uint8), other_t["globals"][k].view(torch.uint8)), (tag, k)
        acc.close()
        ctx.close()


@pytest.mark.parametrize("name", ["ragged_bf16", "wide_odd_bf16", "ragged_f32", "llama_overlap_S8", "gpt_bf16", "llama_bf16_um"])
def test_single_owner_copy_keeps_the_sign_of_zero(lib, name):
    """A parameter with one owner is copied bit for bit (Section 3.3 with a one-term sum): every subnet value is set to
    -0.0, so each single-owner element of the central model must come back with the sign bit set, in every row of the
    tensor and also where subnets that do not hold the block come before the owner in the sum."""
    cfg, S, full_np, full_t, ctx, plan, oplan, fw = _setup(lib, name, seed=13)
    subs = [ctx.twist_extract(plan, fw, s) for s in range(S)]
    for sub in subs:
        for l in range(cfg.n_layers):
            for k in si.layer_shapes(cfg):
                sub.twist_subnet_view(l, k).fill_(-0.0)
    ctx.twist_aggregate(plan, subs, fw)
    torch.cuda.synchronize()
    bits = torch.int16 if cfg.dtype == "bf16" else torch.int32
    checked = 0
    for l in range(cfg.n_layers):
        for k, (kind, axis) in omove.PARTITIONED.items():
            if k not in full_t["layers"][l]:
                continue
            q = cfg.d_head if kind == 0 else cfg.ffn_granule
            single = np.repeat(np.array(oplan[l][kind]["count"]) == 1, q)
            if not single.any():
                continue
            stored_axis = 0 if cfg.out_unit_major and k in si.STORED_TRANSPOSED else axis
            t = full_t["layers"][l][k].view(bits).cpu().numpy()
            sel = t[single] if stored_axis == 0 else t[:, single]
            assert (sel == np.iinfo(sel.dtype).min).all(), (name, l, k)      # sign bit only: -0.0
            checked += sel.size
    assert checked > 0


def test_untrained_partition_roundtrip_is_bit_exact(lib):
    cfg, S, full_np, full_t, ctx, plan, oplan, fw = _setup(lib, "gpt_bf16", seed=6)     # 12 = 4*3 heads, 3072 = 4*768
    before = model_to_numpy(full_t, cfg)
    subs = [ctx.twist_extract(plan, fw, s) for s in range(S)]
    ctx.twist_aggregate(plan, subs, fw)
    after = model_to_numpy(full_t, cfg)
    for l in range(cfg.n_layers):
        for k in before["layers"][l]:
            assert np.array_equal(before["layers"][l][k], after["layers"][l][k]), k
    for k in before["globals"]:
        assert np.array_equal(before["globals"][k], after["globals"][k]), k


@pytest.mark.parametrize("name", ["llama_overlap_S8", "llama_overlap_S8_um"])
def test_aggregate_is_deterministic(lib, name):
    cfg, S, full_np, full_t, ctx, plan, oplan, fw = _setup(lib, name, seed=8)
    subs = [ctx.twist_extract(plan, fw, s) for s in range(S)]
    for s, sub in enumerate(subs):
        _perturb(cfg, sub, s)
    ctx.twist_aggregate(plan, subs, fw)
    first = model_to_numpy(full_t, cfg)
    for l, lw in enumerate(full_np["layers"]):          # reset and repeat
        for k, v in lw.items():
            full_t["layers"][l][k].copy_(torch.tensor(np.ascontiguousarray(_stored(cfg, k, v)), dtype=torch.float64))
    ctx.twist_aggregate(plan, subs, fw)
    second = model_to_numpy(full_t, cfg)
    for l in range(cfg.n_layers):
        for k in first["layers"][l]:
            assert np.array_equal(first["layers"][l][k], second["layers"][l][k])


@pytest.mark.parametrize("name", ["llama_bf16", "llama_bf16_um"])
def test_deployment_extract_leaves_uncovered_units_alone(lib, name):
    cfg, S, full_np, full_t, ctx, plan, oplan, fw = _setup(lib, name, seed=9, require_coverage=False)
    subs = [ctx.twist_extract(plan, fw, s) for s in range(S)]
    for s, sub in enumerate(subs):
        _perturb(cfg, sub, s)
    sub_np = {s: subnet_to_numpy(subs[s], cfg) for s in range(S)}
    want = omove.aggregate(full_np, oplan, sub_np, cfg.d_head, cfg.ffn_granule)
    ctx.twist_aggregate(plan, subs, fw)
    got = model_to_numpy(full_t, cfg)
    cnt = np.array(oplan[0][1]["count"])
    assert (cnt == 0).any()                                 # some neurons really have no owner
    for k in ("w_up", "w_gate"):
        assert np.array_equal(got["layers"][0][k][cnt == 0], full_np["layers"][0][k][cnt == 0])
    assert np.array_equal(got["layers"][0]["w_down"][:, cnt == 0], full_np["layers"][0]["w_down"][:, cnt == 0])
    for k, w in want["layers"][0].items():
        assert rel_fro(got["layers"][0][k], w) <= 5e-3


# ------------------------------------------------------------------------------------------ full-size shapes
@pytest.mark.parametrize("unit_major", [False, True])
def test_workload4_layer_shape_sampled_rows(lib, unit_major):
    """Two layers at the full Llama-7B layer shape, S = 8, in the launch configuration the benchmark times.
    Weights are drawn on the device; the checker recomputes sampled rows and columns from the same values."""
    cfg = replace(si.CFG4, n_layers=2, out_unit_major=unit_major)
    S, hs, fs = 8, 16, 5504
    gen = torch.Generator(device="cuda").manual_seed(4)
    layers = [{k: (torch.randn(shp, generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for k, shp in si.stored_shapes(cfg).items()}
              for _ in range(cfg.n_layers)]
    fw = lib.FullWeights(layers)
    ctx = _ctx(lib, cfg)
    plan = ctx.twist_sample(S, hs, fs, seed=11)
    oplan = sample_plan(cfg.n_layers, cfg.n_heads, cfg.n_ffn_units, S, hs, fs, 11)
    subs = [ctx.twist_extract(plan, fw, s) for s in range(S)]
    rng = np.random.default_rng(0)
    l = 1
    heads = [oplan[l][0]["idx"][s] for s in range(S)]
    units = [np.array(oplan[l][1]["idx"][s]) for s in range(S)]
    # axis along which a stored tensor is cut: the checker's table, except that unit-major storage turns the
    # column cuts of the two output projections into row cuts
    def cut(name):
        ka = omove.PARTITIONED.get(name)
        if ka is None:
            return None
        return (ka[0], 0) if unit_major and name in si.STORED_TRANSPOSED else ka
    # extract: sampled rows / columns of each partitioned tensor are exact copies
    for s in (0, 5, 7):
        e_head = omove.element_index(heads[s], cfg.d_head)
        for name, e in (("wq", e_head), ("wv", e_head), ("w_up", units[s]), ("w_gate", units[s]), ("wo", e_head), ("w_down", units[s])):
            if cut(name)[1] == 0:
                rows = rng.integers(0, len(e), 16)
                got = subs[s].twist_subnet_view(l, name)[torch.tensor(rows).cuda()]
                assert torch.equal(got, layers[l][name][torch.tensor(e[rows]).cuda()]), (s, name)
            else:
                rows = torch.tensor(rng.integers(0, cfg.d_model, 8)).cuda()
                got = subs[s].twist_subnet_view(l, name)[rows]
                assert torch.equal(got, layers[l][name][rows][:, torch.tensor(e).cuda()]), (s, name)
    # train stand-in, then aggregate; check sampled rows against the formula evaluated in fp64
    for s, sub in enumerate(subs):
        for name in si.layer_shapes(cfg):
            v = sub.twist_subnet_view(l, name)
            v.add_((torch.randn(v.shape, generator=gen, device="cuda") * 1e-3).to(v.dtype))
    old = {k: v.clone() for k, v in layers[l].items()}
    ctx.twist_aggregate(plan, subs, fw)
    for name in ("wk", "w_up", "wo", "w_down", "norm1_w"):
        kind_axis = cut(name)
        full_rows = rng.integers(0, layers[l][name].shape[0], 6)
        for r in full_rows:
            r = int(r)
            got = to_numpy(layers[l][name][r])
            if kind_axis is None:
                want = sum(to_numpy(sub.twist_subnet_view(l, name)) for sub in subs)[r] / S
            else:
                kind, axis = kind_axis
                q = cfg.d_head if kind == 0 else 1
                num = np.zeros_like(got)
                den = np.zeros_like(got)
                for s, sub in enumerate(subs):
                    e = omove.element_index(oplan[l][kind]["idx"][s], q)
                    sv = sub.twist_subnet_view(l, name)
                    if axis == 0:
                        pos = np.nonzero(e == r)[0]
                        if len(pos):
                            num += to_numpy(sv[int(pos[0])])
                            den += 1
                    else:
                        num[e] += to_numpy(sv[r])
                        den[e] += 1
                want = np.where(den > 0, num / np.maximum(den, 1), to_numpy(old[name][r]))
            assert rel_fro(got, want) <= 5e-3, (name, r)
            assert bf16_ulp_distance(got, si.to_bf16_grid(want)).max() <= 1, (name, r)
    # counts: Alg. 1 covers every unit, and the counts add up
    _, _, cnt = plan.twist_plan_view(l, 1)
    assert int(cnt.min()) >= 1 and int(cnt.sum()) == S * fs
