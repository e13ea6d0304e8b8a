"""MI355X-native block-wise denoising stage (DualParal hot path) behind a C-ABI library.

`paper_2505_21070_amd.binding` wraps libdualparal.so; `synth` holds the seeded
input generators.  Importing the package loads nothing native.
"""
