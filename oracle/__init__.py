"""CPU oracle of the DQN hot path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this package.  It shares
no code with the HIP library and never imports it.
"""
