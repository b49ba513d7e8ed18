"""CPU oracle of MTAD / MMTAD (arXiv 2407.09722): TEST INFRASTRUCTURE, not product code.

A plain, slow numpy implementation (float64 unless stated) of what the hot path
computes, written from the paper: beam sampling on the auxiliary model (Section 2.1,
Eq. 2), single-pass verification by the target model (Section 3.2, Algorithm 1;
Section 3.3 for the multi-candidate tree), joint-likelihood acceptance of the longest
passing prefix, the bonus token, and the decoding loop (Section 2.2 step 4).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import it.  It
shares no code with the HIP path and does not import it.

Pins (tests/test_oracle_*.py):
  lm.DecoderLM          an independently written decoder from torch library routines
                        (rms_norm, complex-number rotary, scaled_dot_product_attention,
                        silu), float32 and bfloat16 forms; incremental/tree-masked form ==
                        full recompute; causality, rotary shift invariance, sibling order;
                        logit spread closed form.  The decoder architecture itself is fixed
                        by the workload description, not by the paper: "parity unpinned"
                        by the paper for the architecture.
  lm.DecoderLM._rp      hi == library bfloat16(x), lo == library bfloat16(x - hi),
                        |x - (hi + lo)| <= 2^-16 |x|.
  lm.DecoderLM._rkv     == library half precision (range limit 65504 included).
                        Why these two and not one bfloat16 term: the self-noise test
                        (one-term contract: the oracle against a 1e-7 perturbed copy of
                        itself ends more than 2e-2 apart; this contract: below 5e-3).
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
