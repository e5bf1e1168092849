"""MI355X-native sparse snapshot and sparse-to-dense conversion for MoE expert state.

The hot path (snapshot pack / drain, restore unpack, fused Adam replay) runs in the HIP
library ``libmoev.so`` built from ``csrc/``; ``binding`` is its thin ctypes face and
``workloads`` describes the seeded synthetic inputs.  Nothing here falls back to a CPU
implementation: using the binding without the built library raises.
"""
__all__ = ["binding", "workloads"]
