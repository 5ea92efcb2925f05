"""MI355X-native multi-level correlation-volume lookup (block-sparse, MFMA).

`binding` wraps the C-ABI library built from `csrc/`; `synth` draws seeded
synthetic inputs.  Importing the package loads nothing; the first call into
`binding` loads libcorr_mi355x.so and raises if it has not been built.
"""
