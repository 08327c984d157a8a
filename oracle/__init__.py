"""fp64 CPU oracle for circuit evaluation.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It shares no code with the GPU library and neither imports the other.
Parity unpinned: nothing (see tests/test_oracle_pins.py for the pins).
"""
