"""MI355X-native tree-masked Mamba2 SSD verification pass (STree hot path).

``paper_2505_14969_amd.synth``   seeded synthetic inputs (no method arithmetic)
``paper_2505_14969_amd.binding`` ctypes binding of the C-ABI library libstree.so

The HIP library is loaded lazily by ``binding``; importing this package does not
touch the GPU.
"""
__all__ = ["synth", "binding"]
