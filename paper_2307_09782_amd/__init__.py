"""MI355X (gfx950) W4A8 linear-layer path: FP8-E4M3 per-token activations x
FP4-E2M1 group-quantized weights with power-of-two scales, plus LoRC.

``paper_2307_09782_amd.zqfp`` is the thin binding over the C-ABI library
``libzqfp.so`` (built from ``csrc/``); ``paper_2307_09782_amd.inputs`` is the
seeded synthetic-input generator.  Importing the package loads neither.
"""
