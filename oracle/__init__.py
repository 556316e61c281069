"""CPU oracles for prefix-tree decode attention.  TEST INFRASTRUCTURE ONLY.

Nothing in the product package imports this; only ``tests/``, the smoke check
and the benchmark's ``cpu_baseline`` leg do.  Contents:

* ``attention``  - the definition (softmax attention per request over its
  concatenated root-to-leaf context), fp64, plain C behind ctypes.
* ``method``     - the paper's partial-attention / partial-reduction steps
  (Alg. 2-4) in fp64 numpy, to check that tree-merged results equal the
  definition and to replay a task list on the CPU.
* ``planner``    - integer re-derivation of cost estimation, division and
  scheduling, to check the library's plan bit for bit.
"""
