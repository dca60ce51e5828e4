"""libdsqconv for AMD MI355X: b-bit (2..4) quantized convolution on codes.

The compute lives in ``csrc/`` (HIP kernels behind a C ABI declared in
``include/dsqconv.h``); :mod:`paper_1908_05033_amd.binding` only marshals
arguments.  Importing the package does not load the GPU library; the first
call does, and fails loudly if it has not been built.
"""
