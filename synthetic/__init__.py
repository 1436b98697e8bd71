"""Seeded synthetic inputs (weights, latents, labels, VC factors) shared by the
tests, the benchmark and the CPU oracle.  This package holds no arithmetic of
the method itself: it only draws random tensors of the right shapes."""
