"""MI355X-native Multi-Scale Dequant hot path: Python binding over the C-ABI library.

Importing the package does not load the HIP library; the first call into
``paper_2605_13915_amd.binding`` does, and raises if it has not been built.
"""
__all__ = ["binding", "synth"]
