"""CPU oracle for the DARIS hot path -- TEST INFRASTRUCTURE, never a product path.

`forward`  : direct-loop CNN forward pass (C, double accumulation).
`des`      : discrete-event model of the priority/stage scheduler (pure Python integers).
Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
"""
