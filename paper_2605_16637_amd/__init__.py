"""Placement search of a workflow- and heterogeneity-aware LLM scheduler on
MI355X: a C-ABI library of HIP kernels (``csrc/``), a thin ctypes binding
(``binding``) and seeded synthetic rounds (``synth``)."""
__all__ = ["binding", "synth"]
