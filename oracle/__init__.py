"""CPU oracle for the W8A8 + step-cache + variance-compensation DiT sampler.

TEST INFRASTRUCTURE ONLY.  Plain numpy, float64 arithmetic, no blocking or
fusion: every function follows one definition of the paper (or of the DiT
architecture the paper builds on) and cites it.  Floating-point values that
decide an integer code (quantiser decisions) are taken in float32, the
precision the device kernels use for the same decision.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may
import this package.  It shares no code with the HIP path and never imports it.
"""
