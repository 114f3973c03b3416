"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle's
timing leg.  This package holds input generation only: no hashing, no kernel
maps, no convolution arithmetic."""
