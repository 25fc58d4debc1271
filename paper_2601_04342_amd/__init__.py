"""MI355X-native Recurrent Hybrid Attention (ReHyAt) forward operator.

``paper_2601_04342_amd.binding`` is the thin ctypes layer over the C-ABI
library ``librehyat.so`` (hand-written HIP kernels for gfx950);
``paper_2601_04342_amd.synth`` generates the seeded synthetic workloads.
"""
__all__ = ["binding", "synth"]
