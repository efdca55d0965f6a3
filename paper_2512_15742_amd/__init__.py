"""MI355X-native forward pass of vector-quantised KAN layers (SHARe-KAN / LUTHAM).

`paper_2512_15742_amd.binding` is the thin ctypes layer over the C-ABI library
(`include/kan.h`); `paper_2512_15742_amd.synth` draws the seeded synthetic
workloads.  Nothing is imported eagerly so that the input generator can be used
without the HIP library being present.
"""
__all__ = ["binding", "synth"]
