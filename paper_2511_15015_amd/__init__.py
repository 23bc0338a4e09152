"""MI355X-native hot path of DynaExq (arXiv 2511.15015): routed MoE expert
forward over a table of stable expert handles, each expert either resident
bf16 or group-quantized int4, plus hotness counting, budget-feasible top-n
selection, the demotion quantizer and handle publication.

``workloads`` draws the seeded synthetic inputs; ``binding`` is the thin
ctypes layer over the C-ABI library built from ``csrc/``.  The binding is
loaded lazily so that the input generators stay importable on their own.
"""
__all__ = ["workloads", "binding"]
