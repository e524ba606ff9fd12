"""CPU oracle for the freeze-boundary training step (test infrastructure only).

This package is the slow, plain reference that the HIP path is checked against.
It is NOT part of the product: only tests, the smoke entry and the benchmark's
cpu_baseline leg may import it.  It shares no code with the HIP library and
never imports the GPU package.
"""
