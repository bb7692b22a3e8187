"""MI355X-native fused ROSAQ linear layer (rotated, mixed-precision weights).

The HIP library is loaded lazily by `paper_2506_13472_amd.binding`; importing
the package itself touches neither the GPU nor the shared library.
"""
__all__ = ["binding", "synth", "build"]
