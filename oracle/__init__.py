"""CPU oracle of MTAD / MMTAD (arXiv 2407.09722): TEST INFRASTRUCTURE, not product code.

A plain, slow numpy implementation (float64 unless stated) of what the hot path
computes, written from the paper: beam sampling on the auxiliary model (Section 2.1,
Eq. 2), single-pass verification by the target model (Section 3.2, Algorithm 1;
Section 3.3 for the multi-candidate tree), joint-likelihood acceptance of the longest
passing prefix, the bonus token, and the decoding loop (Section 2.2 step 4).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import it.  It
shares no code with the HIP path and does not import it.

Pins (tests/test_oracle_*.py):
  lm.DecoderLM          incremental/tree-masked form == full recompute; hand-computed
                        one-layer case; logit spread closed form.  The decoder
                        architecture itself is fixed by the workload description, not by
                        the paper: "parity unpinned" by the paper for the architecture.
  mtad.beam_search      brute force over all |V|^gamma sequences; width 1 == greedy;
                        stochastic width 1 == ancestral sampling (chi-square).
  mtad.verify           tree form == per-branch sequential decoding == enumeration.
  mtad.accept_*         draft == target gives eta = gamma; tau = 0 accepts all; the
                        bound of Theorem 3.6; Theorem 3.7 (tree length >= chain length);
                        exhaustive enumeration on toy tables.
  mtad.bonus_token      empirical frequency vs the target row (chi-square); argmax mode.
  rng                   uniformity chi-square, independence of streams, fixed vectors
                        produced by tests/golden/make_golden.py (oracle only).
"""
