"""CPU oracle for the BlockBatch denoising path.  TEST INFRASTRUCTURE ONLY.

Plain, slow numpy code written from the paper's definitions; it shares nothing with the
HIP library and must never be imported by the product path (only tests, the smoke check
and the benchmark's cpu_baseline leg may use it).

  model.py      masked-diffusion transformer forward (block forward against a cache row,
                full-sequence forward = cache refresh), vocabulary softmax confidence
  policy.py     Eq. 1 commit, block advance, Alg. 2 MergeSync, refresh cadence
  blockbatch.py Alg. 1 as a step-by-step state machine over one request

Parity status: every function is pinned by tests/test_oracle_*.py except the token
trajectory a whole decode produces, which the paper gives no runnable example for:
"parity unpinned" for trajectory-level outputs (they are pinned only through the
per-step pins).
"""
