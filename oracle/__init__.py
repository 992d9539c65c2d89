"""CPU oracle for XOR-friendly binary quantized top-K search.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only the
tests, the smoke check and the benchmark's CPU-baseline leg do.  The oracle shares
no code, table or helper with the HIP path and never imports it.

Two levels:
  * ``oracle.definition`` -- the paper's formulas written out literally (Python
    ints / NumPy), for tiny and medium inputs.
  * ``oracle.scale``      -- the same steps in plain C (``xfbq_oracle.c``) for the
    large workloads; pinned against the definition level.
"""
