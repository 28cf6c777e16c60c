"""CPU oracle (fp64, plain loops) for the vDNN layer-wise training step.

Test infrastructure: only tests/, the smoke check and the benchmark's cpu_baseline leg may
import this package.  It shares no code with the HIP library.
"""
