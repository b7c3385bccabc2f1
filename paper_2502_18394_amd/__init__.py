"""SPECTRE spectral mixer and Prefix-FFT cache for MI355X (gfx950).

The compute lives in ``csrc/`` (hand-written HIP kernels behind the C ABI of
``include/spectre.h``); ``binding`` marshals arguments to it and ``synth`` draws
seeded inputs.  Importing the package does not load the GPU library; the first
call through ``binding`` does, and fails loudly when it has not been built.
"""
