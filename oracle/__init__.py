"""CPU oracle for Hierarchical Speculative Decoding (HSD).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 reference of
what the HIP library computes.  It is written from the paper's definitions
(Sec. 2 speculative-sampling rule, Alg. 1 HSD, Alg. 2 Verify, Thm 3.1,
Thm 3.2, Cor. 4.1, Sec. 4.3 reduction) and shares no code with the HIP path.
Only the tests, the smoke entry and the bench's cpu_baseline leg may import
it; the product path never does.

Modules
  philox      counter-based Philox4x32-10 generator (published algorithm)
  specsample  accept test, fixed-point residual/bonus sampling, Verify (Alg. 2)
  decoder     pre-norm decoder with early exits (RMSNorm, RoPE, GQA attention,
              SwiGLU), flat KV cache, softmax / one-hot distributions
  hsd         HSD recursion (Alg. 1) and the generation loop
  exact       exact enumeration of HSD's output law on toy models (Thm 3.1)
  latency     gamma, Thm 3.2 / Cor. 4.1 latency, exact-with-overshoot
              expectation, hierarchy selection (Sec. 4), Monte-Carlo

Parity pins (see tests/test_oracle_*.py): every function here is pinned to
something other than itself, except the items listed as "parity unpinned":
  - latency rows >= 3 of the paper's two worked tables (the paper estimated
    gamma empirically, the printed values cannot be regenerated from the text).
"""
