"""Seeded synthetic inputs shared by the oracle's tests, the GPU tests and the benchmark.
Holds memory descriptions and random draws only - none of the engine's arithmetic."""
