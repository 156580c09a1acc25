"""MI355X-native BLOOM block-span forward pass (Petals server hot path).

`paper_2209_01188_amd.binding` wraps the C-ABI library; `synth` draws the seeded
synthetic inputs.  Importing the package loads nothing: the shared library is
opened on first use and its absence is an error, never a fallback.
"""
