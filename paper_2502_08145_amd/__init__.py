"""MI355X-native FC-layer GEMMs (forward, backward-data, backward-weight).

`from paper_2502_08145_amd import binding` gives the Python face of the C-ABI
library; `synth` makes seeded inputs.  Importing the package loads nothing.
"""
