"""MI355X-native d2Cache selective-refresh decoding step (HIP kernels behind a C ABI).

`workloads` (seeded synthetic inputs) imports without the compiled library;
`binding` loads the shared library and fails loudly if it has not been built.
"""
__all__ = ["workloads", "binding"]
