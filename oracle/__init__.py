"""CPU oracle for the HetSeq data-parallel training step (test infrastructure only).

Everything under this package is a plain, slow NumPy implementation of what the
HIP library computes.  It is test infrastructure: only the test-suite, the smoke
check and the benchmark's CPU-baseline leg may import it.  It shares no code,
tables or helpers with the HIP path and never imports it.
"""
