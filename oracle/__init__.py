"""fp64 CPU oracle for the MACE symmetric tensor contraction.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its
Python binding) may import this package; only tests, the smoke check and the
benchmark's cpu_baseline leg use it.  It shares no code, tables or constants
with the HIP path: the coupling tensors here come from the null space of the
rotation generators, the HIP library derives its own from Wigner 3j symbols.

Modules
-------
coupling              real-basis rotation generators, Wigner-D matrices and the
                      SO(3)-invariant three-irrep coupling tensors C(l1,l2,l3).
symmetric_contraction path enumeration, dense generalized coupling tensors U,
                      forward (Algorithm 2 of the paper) and its analytic backward.

Pin status: every function of both modules is pinned by tests/test_oracle_*.py
(closed forms, textbook real spherical harmonics, sympy's Wigner 3j as an
outside library, rotation equivariance, brute-force loops, finite differences).
Absolute values against the MACE / e3nn packages are "parity unpinned": those
packages are not available and the paper prints no numeric example.
"""
