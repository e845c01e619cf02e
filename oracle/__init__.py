"""CPU oracle for the Ozaki-scheme DGEMM (test infrastructure, not part of the product).

A plain, slow, step-by-step implementation of what the paper's method computes, written
from the paper's Section 3 (Eq. 1-3 constants, Eq. 4-8 slicing, Eq. 9-11 error-free
identities), Section 4.2 (integer emulation of FP64 addition) and Section 4.3
(inner-product-wise blocking).  It shares no code with the HIP path: only `tests/`, the
smoke check and the benchmark's CPU-baseline leg may import it.

Modules
-------
formats       Type2 encodings (OCP FP8 E4M3 byte codes, IEEE binary16), written from the format definitions.
ozaki_oracle  constants, slicing, slice-pair products, FP64 accumulation (the plain term-by-term rule and its two
              named variants), blocked driver.
softfloat     ctypes loader of fp64_soft_add.c and fp64_soft_mul.c (IEEE binary64 addition and multiplication
              from their definitions, integer-only).
exact         exact (big-integer) products and the two error measures used in the reports.

Parity status: every function is pinned by the `-m "not gpu"` tests (Table 2 values, exact
reconstruction, exact big-integer products, host-FPU agreement, closed forms, and a product worked
by hand on which the accumulation rules differ, tests/golden/accumulation_rules_2x2x3.txt).
"""
