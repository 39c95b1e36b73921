"""CPU oracle for the HieraSparse hot path. TEST INFRASTRUCTURE ONLY.

Nothing on the product path may import this package: only tests/, the smoke
check and the benchmark's cpu_baseline leg use it. It shares no code with the
HIP library and never imports it.
"""
