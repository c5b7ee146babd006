"""CPU oracle for the PILC entropy-coding stage.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this package: it exists so that the
test-suite, the smoke check and the benchmark's cpu_baseline leg can compare
the GPU library against a plain, slow, obviously-correct implementation.
It shares no code with the HIP path.
"""
