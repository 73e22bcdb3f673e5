"""CPU oracle for the StragglAR AllReduce hot path (arXiv 2505.23523).

THIS PACKAGE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
NumPy implementation used only to check the HIP library.  Only the test
suite, the smoke check and the `cpu_baseline` leg of the benchmark may import
it; the product path never does, and it imports nothing from the product.

What it holds
-------------
* `schedule`  - the schedules as the paper defines them: the completion
  rounds of Alg. 1 (power-of-two n), a ring ReduceScatter among the n-1
  on-time ranks (the "precondition" of Sec. 3.1), and the classic ring
  AllReduce of App. E.  Output: per-round lists of (src, dst, chunk, op).
* `replay`    - applies such a schedule op by op, in order, to n host
  buffers (int32 / fp32 / bf16 with per-op round-to-nearest-even).
* `reference` - results that do not depend on any schedule: the fp64 sum
  (the AllReduce postcondition of Sec. 3.1) and the fold-order closed form
  of the schedule-ordered floating-point result.
* `bf16`      - bfloat16 <-> float32 conversion (round to nearest even).

Parity status: every function here is pinned by the CPU tests against
something outside itself (Thm. 1 round counts, Lemma 1 / invariant I(r)
cardinalities, the Fig. 3b constraint, Table 1 costs, brute-force sums,
a library bf16 conversion); nothing is "parity unpinned".
"""

COPY = 0
REDUCE = 1
REDUCE_EXCHANGE = 2

OP_NAMES = {COPY: "COPY", REDUCE: "REDUCE", REDUCE_EXCHANGE: "REDUCE_EXCHANGE"}
