"""Pins for the checker's generator and Algorithm 1 (Section 3.1)."""
import itertools
import os
from collections import Counter

import pytest

from oracle.rng import Stream, mix
from oracle.sample import ConstraintError, generate_blueprint, inverse_and_count, sample_plan

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_splitmix_published_vector():
    want = [int(x) for x in open(os.path.join(GOLD, "splitmix64_seed1234567.txt")) if not x.startswith("#")]
    s = Stream(0, raw_state=1234567)
    assert [s.u64() for _ in range(5)] == want


def test_stream_keys_differ():
    firsts = {Stream(seed, r, l, k).u64() for seed, r, l, k in itertools.product(range(3), range(3), range(3), range(2))}
    assert len(firsts) == 54
    assert mix(0) == 0  # the finaliser fixes 0; keys are still distinct because the step adds the odd constant


def test_below_is_uniform_and_in_range():
    s = Stream(7)
    n = 6
    c = Counter(s.below(n) for _ in range(60000))
    assert set(c) == set(range(n))
    chi2 = sum((c[i] - 10000) ** 2 / 10000 for i in range(n))
    assert chi2 < 25.7  # chi^2_5 at p = 1e-4


def test_shuffle_all_permutations_equally_likely():
    c = Counter()
    s = Stream(11)
    for _ in range(24000):
        a = [0, 1, 2, 3]
        s.shuffle(a)
        c[tuple(a)] += 1
    assert len(c) == 24
    chi2 = sum((v - 1000) ** 2 / 1000 for v in c.values())
    assert chi2 < 60.0  # chi^2_23 at p ~ 4e-5


def test_unique_choice_every_subset_equally_likely():
    c = Counter()
    s = Stream(13)
    for _ in range(20000):
        c[tuple(sorted(s.unique_choice([0, 1, 2, 3, 4], 2)))] += 1
    assert len(c) == 10
    chi2 = sum((v - 2000) ** 2 / 2000 for v in c.values())
    assert chi2 < 36.0  # chi^2_9 at p ~ 4e-5


@pytest.mark.parametrize("n_full,S,n_sub,common", [
    (12, 4, 3, []), (12, 4, 6, []), (12, 4, 6, [0, 5]), (16, 4, 8, []), (11, 3, 5, [2]), (512, 2, 256, []),
    (7, 3, 7, []), (5, 1, 5, []), (64, 8, 32, [1, 2, 3]),
])
def test_algorithm1_postconditions(n_full, S, n_sub, common):
    for seed in range(5):
        A = generate_blueprint(n_full, S, n_sub, common, Stream(seed, 0, 0, 0))
        assert len(A) == S
        covered = set()
        for row in A:
            assert len(row) == n_sub and row == sorted(row) and len(set(row)) == n_sub
            assert set(common) <= set(row)
            assert all(0 <= b < n_full for b in row)
            covered |= set(row)
        assert covered == set(range(n_full))          # every block is trained by someone
        inv, count = inverse_and_count(A, n_full)
        assert sum(count) == S * n_sub
        assert all(count[b] == S for b in common)
        for s, row in enumerate(A):
            for k, u in enumerate(row):
                assert inv[s][u] == k
            assert sum(1 for x in inv[s] if x >= 0) == n_sub


@pytest.mark.parametrize("n_full,S,n_sub", [(512, 2, 256), (4, 2, 2), (3072, 4, 768), (12, 4, 3)])
def test_tight_bound_gives_exact_partition(n_full, S, n_sub):
    A = generate_blueprint(n_full, S, n_sub, [], Stream(0, 0, 0, 1))
    allb = [b for row in A for b in row]
    assert sorted(allb) == list(range(n_full))


def test_bound_rejection():
    with pytest.raises(ConstraintError):
        generate_blueprint(12, 4, 2, [], Stream(0))            # 12 > 4*2
    with pytest.raises(ConstraintError):
        generate_blueprint(12, 4, 13, [], Stream(0))           # N_sub > N_full
    with pytest.raises(ConstraintError):
        generate_blueprint(12, 4, 4, [0, 1], Stream(0))        # 10 > 4*(4-2)
    generate_blueprint(12, 4, 6, [0, 1, 2], Stream(0))         # 9 <= 4*3: allowed
    # the bound is exactly (N_full + (S-1)|C|)/S <= N_sub
    for n_full, S, c in itertools.product(range(1, 9), range(1, 4), range(0, 3)):
        if c > n_full:
            continue
        for n_sub in range(max(c, 1), n_full + 1):
            ok = (n_full + (S - 1) * c) <= S * n_sub
            try:
                generate_blueprint(n_full, S, n_sub, list(range(c)), Stream(1))
                assert ok
            except ConstraintError:
                assert not ok


def test_inclusion_frequency_is_uniform():
    # every non-common block must be in a given subnet with probability N_sub / N_full
    n_full, S, n_sub, trials = 6, 3, 4, 6000
    hits = [[0] * n_full for _ in range(S)]
    for seed in range(trials):
        A = generate_blueprint(n_full, S, n_sub, [], Stream(seed, 3, 1, 0))
        for s, row in enumerate(A):
            for b in row:
                hits[s][b] += 1
    p = n_sub / n_full
    sd = (trials * p * (1 - p)) ** 0.5
    for s in range(S):
        for b in range(n_full):
            assert abs(hits[s][b] - trials * p) < 4.5 * sd, (s, b, hits[s][b])


def test_deployment_mode_single_subnet():
    # relaxed constraints: one subnet, no coverage requirement, any size <= N_full
    seen = Counter()
    for seed in range(3000):
        A = generate_blueprint(12, 1, 4, [0], Stream(seed), require_coverage=False)
        assert len(A) == 1 and len(A[0]) == 4 and A[0] == sorted(set(A[0])) and 0 in A[0]
        seen.update(A[0])
    assert seen[0] == 3000
    for b in range(1, 12):
        assert abs(seen[b] - 3000 * 3 / 11) < 4.5 * (3000 * (3 / 11) * (8 / 11)) ** 0.5


def test_plan_streams_and_shared_layers():
    plan = sample_plan(4, 12, 12, 4, 6, 6, seed=5, layer_shared=[1, 0, 0, 1])
    assert plan[0][0]["idx"] == [list(range(12))] * 4 and plan[0][0]["n_sub"] == 12
    assert plan[3][1]["count"] == [4] * 12
    assert plan[1][0]["idx"] != plan[2][0]["idx"]          # independent stream per layer
    assert plan[1][0]["idx"] != plan[1][1]["idx"]          # and per kind
    again = sample_plan(4, 12, 12, 4, 6, 6, seed=5, layer_shared=[1, 0, 0, 1])
    assert again[1][0]["idx"] == plan[1][0]["idx"]         # deterministic
    other = sample_plan(4, 12, 12, 4, 6, 6, seed=5, rnd=1, layer_shared=[1, 0, 0, 1])
    assert other[1][0]["idx"] != plan[1][0]["idx"]         # resampled each round
