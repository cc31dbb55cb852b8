"""TensorGRaD optimizer hot path for AMD MI355X (gfx950).

`paper_2501_02379_amd.tgrad` is the ctypes binding over the C-ABI library
(`libtgrad.so`, built from `csrc/`); `paper_2501_02379_amd.synth` draws the
seeded synthetic inputs.  Importing the package loads nothing native; the
binding raises when the library is missing.
"""
