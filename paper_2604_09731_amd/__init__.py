"""MI355X-native tree-verification hot path of SMART speculative decoding.

`paper_2604_09731_amd.binding` wraps the C-ABI library (loaded lazily, fails
loudly when it has not been built); `paper_2604_09731_amd.workloads` holds the
seeded synthetic input generators.
"""
__all__ = ["binding", "workloads"]
