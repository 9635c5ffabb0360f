"""KV-cache merging compression pass for AMD MI355X: HIP kernels behind a C ABI.

`binding` loads libkvm.so lazily on first use and raises if it is missing; `synth`
holds the seeded workload generators (no arithmetic of the method).
"""
__all__ = ["binding", "synth", "build"]
