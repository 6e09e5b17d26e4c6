"""MI355X-native quantized LoRA linear layer (forward and backward).

The HIP library is loaded lazily by :mod:`paper_2306_08162_amd.binding`;
importing the package (or :mod:`workloads`) does not need a GPU.
"""

__all__ = ["binding", "workloads"]
