"""CPU oracle for the W4A4 static-quantized linear path (test infrastructure only).

Nothing in the product path may import this package: it exists so that the tests, the
smoke check and the benchmark's cpu_baseline leg have an independent, slow, obviously
correct answer to compare the HIP library with.
"""
