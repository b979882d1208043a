"""Sampled mini-batch preparation (neighbour sampling -> MFG blocks -> feature gather) on MI355X.

`paper_2110_08450_amd.binding` wraps the C-ABI library built from `csrc/`; it is loaded on first
use and raises if the library is missing.  `paper_2110_08450_amd.synth` makes the seeded
synthetic inputs.
"""
