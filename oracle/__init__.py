"""CPU oracle for the module-parallel local step.  TEST INFRASTRUCTURE ONLY.

Imported by tests/, by the smoke check and by the benchmark's cpu_baseline leg; the
product path (the HIP library and its binding) never imports it.
"""
