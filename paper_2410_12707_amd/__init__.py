"""MI355X-native AdaTopK compress / decompress (hand-written HIP behind a C ABI).

``workloads`` draws the seeded synthetic inputs; ``binding`` marshals torch device
tensors into the C-ABI library ``libadatopk.so`` built from ``csrc/``.  Nothing here
falls back to a CPU implementation: a missing library raises on first use.
"""
__all__ = ["workloads", "binding", "build"]
