"""AdaCGD hot path for MI355X: hand-written HIP kernels behind a C ABI.

`workloads` (seeded synthetic inputs) imports without the native library;
`engine` loads the library on first use and raises if it has not been built.
"""
__all__ = ["workloads", "engine"]
