"""MI355X-native local attention for one device's share of the BurstAttention ring.

`binding` wraps the C-ABI library built from `csrc/`; `workloads` holds the seeded
synthetic input generators (no attention arithmetic).
"""
__all__ = ["binding", "workloads"]
