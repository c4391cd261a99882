"""CPU oracle for the GSPMD per-partition einsum path.  TEST INFRASTRUCTURE ONLY:
imported by tests/, the smoke check and bench.py's cpu_baseline leg, never by
the product package.  It shares no code with the HIP library."""
