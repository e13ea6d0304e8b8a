"""CPU oracle for the block-wise denoising stage.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain reference that the
GPU library is checked against.  Only tests, the smoke check and the bench's
CPU-baseline leg may import it; the product package never does, and nothing in
here imports the product package.
"""
