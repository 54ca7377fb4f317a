"""MI355X-native hot path of Cartridge / Self-Study training (arxiv 2506.06266).

`binding` holds the ctypes wrappers over the C-ABI library built from `csrc/`;
`synth` holds the seeded input generators.  Nothing is loaded at import time.
"""
__all__ = ["binding", "synth"]
