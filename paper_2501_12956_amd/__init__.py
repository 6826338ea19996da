"""MI355X-native GANQ per-layer solver: thin Python binding over the C-ABI library.

Importing the package loads nothing; ``paper_2501_12956_amd.binding`` loads the
HIP library on first use and raises if it has not been built.
"""
__all__ = ["binding", "synth"]
