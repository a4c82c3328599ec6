"""CPU oracle of the OCS-expanded quantized layer: test infrastructure, not product code.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
"""
