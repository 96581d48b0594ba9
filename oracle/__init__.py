"""CPU oracle of the ANPD verification path.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may
import this package.  It shares no code with the HIP library and never
imports it.
"""
