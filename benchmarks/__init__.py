"""Measurement scripts beside bench.py (not part of the library): whole cycles, the widened entry
points, and attention / verify-accept at the larger configurations.  Run from the repository root,
e.g. `python -m benchmarks.configs_bench`."""
