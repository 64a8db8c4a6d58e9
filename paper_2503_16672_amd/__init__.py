"""2:4-activation-sparse Squared-ReLU FFN for MI355X (gfx950): HIP kernels behind a C-ABI library.

`paper_2503_16672_amd.ffn24` is the thin binding over the shared library; `synth` draws the seeded
synthetic inputs.  Importing the package does not load the library; the first call does, and fails
loudly if it has not been built.
"""
