"""MI355X-native hot path of the Based sequence mixer (arXiv 2402.18668).

``paper_2402_18668_amd.based`` binds the C-ABI HIP library (``csrc/``); ``synth`` holds the
seeded synthetic inputs.  The binding is imported lazily so that CPU-only tools can use
``synth`` without the built library.
"""
__all__ = ["synth"]
