"""CPU oracle of the DoRA module hot path.  TEST INFRASTRUCTURE ONLY.

Only the tests, `__graft_entry__.smoke()` and the bench's `cpu_baseline` leg may
import this package.  It imports nothing from the HIP path.
"""
