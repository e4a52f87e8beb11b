"""MI355X-native OmniSparse hot path: thin Python binding over the C-ABI HIP library.

Importing the package loads nothing; `paper_2511_12201_amd.binding` loads the
built shared library on first use and raises if it is missing.
"""
__all__ = ["binding", "synth", "build"]
