"""MI355X-native SliceMoE expert-FFN hot path (HIP kernels behind a C-ABI library).

Importing the package loads nothing heavy; `paper_2512_12990_amd.binding` loads the built
library and fails loudly when it is missing.
"""
__all__ = ["binding", "synth"]
