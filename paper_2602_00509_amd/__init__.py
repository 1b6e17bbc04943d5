"""MI355X-native hot path of one GPU's share of an expert-parallel MoE layer
(PROBE, arxiv 2602.00509): top-k gate, lookahead predictor, plan-driven permutation,
grouped SwiGLU FFN, weighted combine.

``probe``     thin ctypes binding of the C-ABI library (libprobe.so, hand-written HIP).
``workload``  seeded synthetic input generators (no layer arithmetic).
"""
__all__ = ["probe", "workload"]
