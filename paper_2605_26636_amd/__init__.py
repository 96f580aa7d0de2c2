"""MI355X-native token mixers of JetViT's hybrid-attention ViT (HIP library + ctypes binding).

`synth` (seeded inputs) imports without the compiled library; `binding` loads
paper_2605_26636_amd/libjetvit.so on first use and raises if it is missing.
"""
__all__ = ["binding", "synth", "build"]
