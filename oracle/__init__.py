"""fp64 CPU oracle of the alpha retention step (test infrastructure only).

Only tests, the smoke entry and the CPU-baseline leg of the benchmark may
import this package.  It shares no code with the HIP library and never
imports it.
"""
