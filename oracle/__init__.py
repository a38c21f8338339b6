"""CPU oracle for the Lagom hot path -- TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct implementations of what the HIP library computes:

* ``collective``  -- reduce-copy / gather-copy local steps and the textbook ring
  collectives composed from them (paper Sec. 2.1 names the collectives; Sec. 3.2
  describes a communication kernel as NC blocks moving data at granularity C).
* ``gemm``        -- C = A.B from bf16 inputs, fp64 reference accumulation.
* ``cost_model``  -- the unified overlap cost model (Eq. 1) over the contention
  wave model (Eq. 4-6).
* ``search``      -- the priority metric H (Eq. 7), the cost-effectiveness loop
  (Alg. 1) with resource-efficient tuning (Alg. 2), and brute-force search.
* ``loops.c``     -- the same copy/reduce/GEMM definitions as plain C loops, used
  only to time the oracle on the host cores.

Nothing here imports, links or shares code with the HIP library or its Python
binding.  Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; the product path never does.

Parity status: every function in this package is pinned by ``tests/test_oracle_*``
against closed forms, library routines, hand-worked fixtures or brute force, except
the absolute accuracy of the cost model (the paper prints no numeric worked
example): its arithmetic is pinned by hand-computed closed forms only --
"parity unpinned" for model-versus-hardware accuracy.
"""
