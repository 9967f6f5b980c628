"""MI355X-native OVGGT streaming hot path: bounded-cache global attention plus
the Self-Selective-Caching update, as HIP kernels behind a C ABI.

`binding` wraps the shared library (and raises if it is not built); `synth`
draws the seeded synthetic streams used by tests and the benchmark.
"""
__all__ = ["binding", "synth"]
