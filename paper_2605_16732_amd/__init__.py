"""MI355X-native rotation-aware W4A4 linear layer (DiRotQ hot path).

`binding` wraps the C-ABI library built from `csrc/`; `inputs` draws the seeded
synthetic workloads; `build` compiles the library.  Importing the package loads
nothing: the library is opened on first use and its absence is an error.
"""
