"""MI355X-native CalibQuant hot path: 1/2-bit KV-cache quantizer and fused decode attention.

`binding` wraps the C-ABI library (HIP kernels); `synth` draws the synthetic workloads.
Nothing here imports the CPU oracle.
"""
__all__ = ["binding", "synth"]
