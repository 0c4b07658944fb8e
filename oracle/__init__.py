"""CPU oracle for the APOLLO / APOLLO-Mini optimizer step (Algorithm 1 of the paper).

This package is TEST INFRASTRUCTURE.  It is a plain, slow, fp64 numpy statement of what the
step computes, written from the paper; it shares no code with the HIP library and must never
be imported by it.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may
use it.

Modules
  philox  -- Philox4x32-10 counter-based generator (Salmon et al., SC'11).
  gauss   -- the fixed fp32 Box-Muller recipe that turns Philox words into N(0,1) variates,
             and the projection matrix P built from them (Algorithm 1, "P_t <- N_seed(0,1/r)").
  apollo  -- the step itself (Algorithm 1; low-rank moments and scaling factor of
             Section 4.1; tensor-wise factor of Section 4.2; norm-growth limiter of Section 3.2).
  q8      -- group-wise 8-bit weight storage (Section 5.4 / Table 6: 8-bit integer weights,
             groups of 128) and the stochastic rounding of its codes.
  adamw   -- element-wise AdamW (Section 3.1, Eq. 1, with decoupled weight decay) for the
             parameters that are not projected (embeddings, norm gains, output head).

Pin status: every function here is pinned by tests that run without a GPU (known-answer
vectors, exact rational arithmetic, closed forms, brute force, statistical laws).  The one
thing nothing can pin is a whole training trajectory on language-model data: the paper prints
no intermediate values -- "parity unpinned" for that, and only for that.
"""
