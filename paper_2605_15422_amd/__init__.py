"""MI355X-native shared-prompt (DualKV) attention: HIP kernels behind a C ABI.

``workloads`` (seeded synthetic inputs) imports without the compiled library;
everything that computes lives in ``binding`` and fails loudly if
``libdualkv.so`` has not been built.
"""
__all__ = ["workloads", "binding", "accounting"]
