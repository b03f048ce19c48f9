"""MI355X-native binary-layer kernels (BMXNet hot path): thin Python binding over libbmx.

``paper_1705_09864_amd.binding`` marshals torch device tensors into the C ABI of
``include/bmx.h``; ``paper_1705_09864_amd.synth`` draws the seeded synthetic inputs;
``paper_1705_09864_amd.build`` compiles the HIP sources for gfx950.
"""
