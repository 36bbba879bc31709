"""TEST INFRASTRUCTURE - CPU oracle of the integer softmax / GELU / requantization.

Importable only from tests, the smoke check and the benchmark's cpu_baseline leg.
"""
