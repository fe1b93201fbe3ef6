"""MI355X-native sparse MoE layer (router, activation counts, next-layer
prediction, permute, grouped SwiGLU experts, combine) behind a C ABI.

``paper_2501_10375_amd.moe`` is the thin ctypes binding over the HIP library;
``paper_2501_10375_amd.synth`` makes seeded synthetic inputs.  Importing the
package loads neither: the binding loads the shared library on first use and
raises if it has not been built.
"""
__all__ = ["moe", "synth"]
