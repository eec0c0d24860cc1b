"""CPU oracle for one rank's ZeRO training step and Poplar's profiling/allocation.

TEST INFRASTRUCTURE ONLY.  Everything in this package is a plain, slow,
fp64 NumPy statement of what the GPU path must compute.  It shares no code
with the HIP library or its Python binding, and nothing in the product path
may import it: only the tests, the smoke check and the CPU-baseline leg of
the benchmark do.

Modules
-------
transformer : GPT-2 / Llama decoder layer and whole-model forward/backward
              (textbook definitions; the paper runs stock models and fixes
              none of their internals).
optimizer   : Adam and the ZeRO shard index arithmetic (Appendix "Details
              about ZeRO"), local gradient reduction and parameter gather.
spline      : natural cubic spline (Appendix "Cubic Spline Interpolation").
profiling   : TimeConsumedDuringStep per ZeRO stage (Section "Time Consumed
              Estimation") and the max-batch search of Algorithm 1.
allocate    : Algorithm 2, both branches, with Eq. (1)-(4) of the problem
              formulation.

Parity status: every function is pinned by tests/test_oracle_*.py against
finite differences, closed forms, library routines or brute force, except
where a header says "parity unpinned".
"""
