"""MI355X-native forward pass of one EdgePipe pipeline stage (a contiguous run
of ViT encoder layers on a micro-batch) and the paper's layer-to-device
partition planner, behind a C-ABI library.

Importing the package loads nothing; `paper_2110_14895_amd.binding` opens the
shared library on first use and raises if it has not been built.
"""
__all__ = ["binding", "synth"]
