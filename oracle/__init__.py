"""CPU oracle for the MuLo-SD parallel verification step.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct
CPU statement of what the verification step computes (numpy / torch-CPU,
float64 unless a rounding point is stated).  It shares no code with the HIP
library and never imports it.  Only the test-suite, the smoke check and the
benchmark's cpu-baseline leg may import it; the product path never does.

Modules (each function cites the passage of the paper it follows):
  philox    counter-based uniforms (the paper names no generator; Philox4x32-10,
            Salmon et al. SC'11, is this build's choice)
  upsample  Step 2: draft tokens / distributions onto the target grid (Sec. 3.2)
  decoder   Step 3: target forward over the draft block against a KV cache; single-token queries at
            scattered cache rows with a per-query set of visible rows (island-parallel re-sampling)
  accept    Step 4: softmax, pooled mass (Eq. 3), accept test (Eq. 1)
  local     Step 5: local neighbourhood expansion (Eq. 6-7)
  resample  residual resampling (Eq. 2) through an integer CDF
  step      the whole verification step (Alg. 1 Steps 2-5 + one-shot resample); sequential re-sampling
            (Alg. 1 Step 6); island-parallel re-sampling (Sec. 3.4)

Pin status (see tests/test_oracle_*.py):
  upsample, accept, local, resample, step : pinned (invariants, closed forms,
      brute force, exact enumeration).
  decoder : structure pinned (causality, textbook special cases, float64
      triple-loop pieces); the logit VALUES for random weights have no external
      reference -> "parity unpinned" for the values themselves.
  philox  : pinned: the three published known-answer vectors of Philox4x32-10 (tests/golden/), and
      uniformity / independence / avalanche statistically.
  step.resample_islands : pinned as far as the paper fixes it (one island from t0 on = sequential
      re-sampling, itself pinned as ancestral sampling; one target call per rank; draws are inverse-CDF
      draws of the rows produced; stale cache rows of pending positions never reach a result).  WHICH
      earlier positions a concurrently evaluated query may attend to is a reading of Sec. 3.4 (settled
      positions only), not something the paper states: that choice is "parity unpinned".
"""
