"""CPU oracle for the tensor-tiling execution path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 / exact-integer implementations written from the paper
(arXiv 1805.04170) to check the HIP library against.  Nothing in the product
package imports this; only tests, the smoke check and the benchmark's
cpu_baseline leg do.  It shares no code with the HIP path.

Modules
  tiling   - k-cut tiling geometry, tile / untile / retile      (Sec. 4.1, Thm. 2)
  layers   - untiled fp64 FC and convolution forward / backward  (Sec. 2.1), through numpy
  layers_plain - the same operators as plain nested loops (C code in layers_plain.c): the definitions written out,
             which pin `layers` and which the benchmark's cpu_baseline times
  execute  - aligned forms, per-shard execution, reduction       (Sec. 4.2.1, Sec. 5.2)
  cost     - conversion costs, Eq. (2), Algorithm 1, brute force (Sec. 4.2-4.3; C code in cost.c)
  naive_comm - the closed-form volumes of the worked MLP example (Sec. 2.2)
  graph    - cost and exhaustive search on a general dataflow graph: d-dimensional tensors, contractions,
             element-wise and batch-only operators (Sec. 4.5)

Parity pins: every function here is pinned by tests/test_oracle_*.py except
the k>1 cost model, whose only pins are closed forms, the k=1 physical traffic
count and brute force of the same reading ("parity unpinned by the paper"
beyond those; see cost.py).
"""
