"""CPU fp64 oracle of the elastic selective training step.  TEST INFRASTRUCTURE ONLY.

Plain numpy float64 code written from the paper's definitions: forward and
masked backward passes, tensor importance, the time model and the tensor
selection, and the optimizer formulas.  It shares no code with the HIP
library and must never be imported by the product path; only the tests, the
smoke check and the benchmark's CPU-baseline leg use it.
"""
