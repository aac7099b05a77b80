"""CPU oracle for the SWARM pipeline-stage hot path (test infrastructure only).

Nothing under this package is part of the product: only the tests, the smoke
check and the benchmark's cpu_baseline leg may import it.  It shares no code
with the HIP library and never imports it.
"""
