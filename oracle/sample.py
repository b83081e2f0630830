"""Subnet generator: Algorithm 1 ("Generate Training Subnet Blueprint") and its deployment variant.

Test infrastructure (see the package docstring).  Follows Section 3.1 in the paper's notation:
N_full blocks, S subnets, N_sub blocks per subnet, common set C, blueprint A (S x N_sub).

Readings where the text is silent (all also listed in the design notes):
  * C' (never defined) is the complement of C, randomly permuted, since the section says the
    subnets are drawn uniformly at random while nothing else in that loop is random.
  * A's unassigned slots do not count as "filled" (rows are kept as sets of assigned blocks here).
  * N_empty = 0 means "nothing to top up".
  * unique_choice draws uniformly without replacement from the ascending complement of the row.
  * deployment ("we relax our constraints"): no coverage pass; each row is C plus a uniform
    draw from the complement of C.
"""
from .rng import Stream

KIND_HEAD, KIND_FFN = 0, 1


class ConstraintError(ValueError):
    """The size bound (N_full + (S-1)|C|)/S <= N_sub <= N_full of Section 3.1 is violated."""


def generate_blueprint(n_full, S, n_sub, common, stream, require_coverage=True):
    C = list(common)
    if sorted(set(C)) != C or any(b < 0 or b >= n_full for b in C):
        raise ValueError("common set must be sorted, unique and within [0, N_full)")
    c = len(C)
    if S < 1 or n_sub < 1 or n_sub > n_full or n_sub < c:
        raise ConstraintError("need |C| <= N_sub <= N_full")
    if require_coverage and n_full - c > S * (n_sub - c):
        raise ConstraintError("N_full - |C| <= S (N_sub - |C|) violated")

    # Each subnet's blueprint row is kept as a membership set: what matters about A[s, :] is which blocks it names
    # (the row is returned in ascending order, so slot positions carry no information).
    members = [set(C) for _ in range(S)]                     # every subnet holds the common blocks
    if require_coverage:
        # coverage: the blocks outside C, in random order, are dealt to the subnets in turn, one block each per turn,
        # so every block is trained by exactly one subnet before anything is drawn freely
        rest = [b for b in range(n_full) if b not in members[0]]
        stream.shuffle(rest)
        for turn, b in enumerate(rest):
            members[turn % S].add(b)
    for s in range(S):
        # top-up: whatever the subnet still lacks is drawn uniformly, without replacement, from the blocks it does not hold
        lacking = n_sub - len(members[s])
        if lacking > 0:
            outside = [b for b in range(n_full) if b not in members[s]]
            members[s].update(stream.unique_choice(outside, lacking))
    return [sorted(m) for m in members]


def inverse_and_count(A, n_full):
    """inv[s][u] = position of block u in row s (or -1); count[u] = number of rows holding u
    (the denominator of the aggregation formula of Section 3.3)."""
    inv = [[-1] * n_full for _ in A]
    count = [0] * n_full
    for s, row in enumerate(A):
        for k, u in enumerate(row):
            inv[s][u] = k
            count[u] += 1
    return inv, count


def sample_plan(n_layers, n_heads, n_ffn_units, S, heads_sub, ffn_units_sub, seed, rnd=0,
                common_heads=(), common_ffn=(), layer_shared=None, require_coverage=True):
    """One blueprint per (layer, kind), each from its own stream keyed (seed, round, layer, kind).

    A layer flagged shared keeps every block in every subnet (N_sub = N_full, identity rows),
    as the experiments do for the first and last layers (Section 5, "Setup").
    Returns plan[layer][kind] = {"idx": A, "inv": inv, "count": count, "n_full":, "n_sub":}.
    """
    plan = []
    for l in range(n_layers):
        per_kind = []
        for kind, n_full, n_sub, common in ((KIND_HEAD, n_heads, heads_sub, common_heads),
                                            (KIND_FFN, n_ffn_units, ffn_units_sub, common_ffn)):
            if layer_shared is not None and layer_shared[l]:
                A = [list(range(n_full)) for _ in range(S)]
                n_sub_l = n_full
            else:
                A = generate_blueprint(n_full, S, n_sub, common, Stream(seed, rnd, l, kind), require_coverage)
                n_sub_l = n_sub
            inv, count = inverse_and_count(A, n_full)
            per_kind.append({"idx": A, "inv": inv, "count": count, "n_full": n_full, "n_sub": n_sub_l})
        plan.append(per_kind)
    return plan
