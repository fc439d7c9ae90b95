"""Seeded synthetic input generators.  They serve the GPU library's tests, the
benchmark and the CPU checker alike, and hold none of the method's arithmetic:
importing this package imports neither of the two."""
