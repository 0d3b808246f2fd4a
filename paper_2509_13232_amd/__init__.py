"""MI355X-native hot path of Single-stream Policy Optimization (arXiv 2509.13232).

The arithmetic lives in the HIP library ``libspo_hip.so`` built from ``csrc/``;
``binding`` marshals torch tensors into its C entry points (same names).
``workloads`` draws the synthetic benchmark inputs and touches neither.
The library is loaded on first use and its absence is an error: there is no
CPU or PyTorch fallback.
"""

__all__ = ["binding", "workloads"]
