"""cgtp: Clebsch-Gordan tensor products and fused equivariant graph convolution on MI355X.

`paper_2501_13986_amd.binding` is the thin ctypes layer over the C-ABI library built from
`csrc/`; `paper_2501_13986_amd.synth` draws seeded synthetic inputs.  Importing the package
itself loads nothing native; the binding raises if the library is missing.
"""
