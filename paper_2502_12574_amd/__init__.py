"""Head-wise offloaded attention for AMD MI355X (gfx950): thin Python binding over the C-ABI library.

Importing the package loads nothing; `paper_2502_12574_amd.binding` loads libheadinfer.so on first use and
fails loudly if it is missing.  `paper_2502_12574_amd.synth` draws the seeded synthetic inputs.
"""
__all__ = ["binding", "synth", "build"]
