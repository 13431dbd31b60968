"""fp64 CPU oracle for the PRISM hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library or its
Python binding) imports, links or executes anything in this package; only the
tests, the smoke check and the CPU-baseline leg of the benchmark do.  It shares
no code, tables or helpers with the HIP path.

Modules
  gauss_sketch  counter-based Gaussian sketch generator (Philox4x32-10 +
                Box-Muller with fully specified fp64 arithmetic)
  prism_ref     the PRISM iterations (polar factor, coupled square root,
                coupled inverse p-th root) and the sketched coefficient fit

Parity status: every function is pinned by tests/test_oracle_*.py except the
items listed as "parity unpinned" in prism_ref's header.
"""
