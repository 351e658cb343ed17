"""CPU oracle for thread-block-level kernel scheduling (slicing, persistent-worker
preemption, profile-guided configuration choice).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct CPU
statement of what the scheduling path computes.  It shares no code with the HIP
library, never imports it, and must never be imported by the product path: only the
tests, the smoke check and the benchmark's cpu_baseline leg may call it.

Floating point is carried in fp64 and rounded once to the storage type.

Pinning status (see tests/test_oracle_*.py):
  grid / slicing / persistent-worker schedules  pinned (paper's worked examples, brute force)
  saxpy, reduce_sum, gemm, gemv, softmax, layernorm, attn_decode  pinned (closed forms, invariants)
  turnaround estimate (Eq. 1) and selection rule  pinned (closed form, hand-made tables)
  latency / throughput figures                   parity unpinned (measured only)
"""
