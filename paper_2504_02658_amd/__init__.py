"""MI355X-native W3A16 + low-rank expert linear (the inference hot path of MiLo).

The compute lives in the HIP library built from `csrc/`; `api` is the thin ctypes
binding over its C ABI and `workloads` draws the seeded synthetic inputs.
Nothing is imported eagerly so that the input generators stay usable on a
machine where the library has not been built.
"""
__all__ = ["api", "workloads"]
