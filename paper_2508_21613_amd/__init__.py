"""MI355X-native scoring of post-failure execution plans (Chameleon, arXiv 2508.21613).

`paper_2508_21613_amd.binding` is the thin ctypes layer over the C-ABI library libchm.so
(hand-written HIP, gfx950); `paper_2508_21613_amd.synth` holds the seeded input generators.
Importing the package loads neither: import the submodule you need.
"""
__all__ = ["binding", "synth"]
