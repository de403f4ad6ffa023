"""CPU oracle (test infrastructure).

Only tests/, the smoke check and the bench's cpu_baseline leg may import this package.
The HIP library never does, and this package never imports the HIP library.
"""
