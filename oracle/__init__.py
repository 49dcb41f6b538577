"""CPU oracle for the SpQR decode + matvec path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this package: only tests/, the smoke
check and the benchmark's cpu_baseline leg do.  It shares no code with the HIP
library or its Python binding.
"""
