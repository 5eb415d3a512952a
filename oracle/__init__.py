"""CPU oracle of the HiFT step.  Test infrastructure: imported only by the tests, the smoke
check and the benchmark's CPU-baseline leg; never by the GPU library or its binding."""
