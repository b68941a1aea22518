"""CPU oracle for the constant-batch decode step with in-flight weight updates.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, readable restatement of what the
generation engine computes (Alg. 2, Actor loop; Sec. 2.1 eq. 1 for the sampled
distribution; Sec. 2.1 truncated-IS equation for why the behaviour log-prob is recorded;
Sec. 5.1 for the stale-KV semantics of an in-flight update).  It shares no code with the
HIP library and is imported only by tests/, by the smoke check and by the benchmark's
`cpu_baseline` leg.  The product path never calls it.

Model arithmetic is float64 on bf16-rounded weights unless a dtype is passed; the sampler's
integer decision (the arg-max of logits + Gumbel noise) is taken in float32 with the exact
operation order written in `sampler.py`, because the device takes it in float32 too.

Pinned by tests/test_oracle_*.py: every function here is checked against a closed form, a
brute-force recomputation, a library routine on a special case, or published known-answer
vectors.  The paper prints no numeric example for this path, so agreement with *its* numbers is
unpinned; what is pinned is the mathematics.
"""
