"""CPU oracle of the integer-only convolution layer: TEST INFRASTRUCTURE.

Only tests/, the smoke check and the benchmark's CPU-baseline leg may import
this package.  The GPU library shares no code with it.
"""
