"""MI355X-native UNIQUE decode-time top-k sparse attention (page stats, page score, top-k, paged decode).

The compute lives in the HIP library under ``csrc/`` behind the C ABI declared in
``include/unique.h``; ``binding`` is the ctypes layer over it. Nothing is loaded
at import time: ``binding.load()`` opens the built library and raises if it is missing.
"""
__all__ = ["binding", "workloads"]
