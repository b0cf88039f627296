"""MI355X-native local attention for one device's share of the BurstAttention ring.

`binding` wraps the C-ABI library built from `csrc/`; `harness` holds the single-GPU chunk walks
(host orchestration only); `autograd` exposes a walk as one differentiable torch call; `workloads`
holds the seeded synthetic input generators (no attention arithmetic).
"""
__all__ = ["binding", "harness", "autograd", "workloads"]
