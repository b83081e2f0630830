"""CPU checker ("oracle") for the TwIST hot path: sample -> extract -> subnet fwd+bwd -> step -> aggregate.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 numpy written from the paper's definitions.
It shares no code with the HIP library and must never be imported by the product package;
only the tests, the smoke check and the benchmark's CPU-baseline leg may call it.

Parity status of each part (what pins it besides itself):
  rng / sample   structure pinned by Algorithm 1's post-conditions and the size bound of
                 Section 3.1; the bit generator is pinned to SplitMix64's published outputs.
                 WHICH permutation a seed gives is "parity unpinned" with respect to the
                 paper (it names no generator).
  extract        pinned: masked-model equivalence (Section 4.1), Appendix C parameter counts
                 and the communication column of Table 2.
  forward        pinned: textbook transformer via an independent library graph, masked
                 equivalence, Monte-Carlo scale factors (Theorems A.3 and A.7).
  backward       pinned: central finite differences and library autograd.
  step           pinned: closed-form scalar recurrences.
  aggregate      pinned: brute-force evaluation of the aggregation formula of Section 3.3,
                 partition -> concatenation, identical subnets -> mean.
"""
