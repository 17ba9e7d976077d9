"""MI355X-native MoE-instance layer step (Janus, arXiv 2512.13525, Sec. 3.4).

``paper_2512_13525_amd.binding`` is the thin ctypes layer over the C-ABI library
built from ``csrc/``; ``paper_2512_13525_amd.workloads`` draws seeded synthetic
inputs.  Nothing is imported eagerly so that the input generators can be used on a
machine without the built library.
"""
__all__ = ["binding", "workloads"]
