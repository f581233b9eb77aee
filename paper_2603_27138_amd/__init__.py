"""MI355X-native GPU side of GPU-CPU collaborative block-wise sparse decode attention.

`workload` (seeded synthetic inputs) is importable anywhere; `binding` loads the
HIP shared library and fails loudly if it has not been built.
"""
__all__ = ["workload", "binding", "build"]
