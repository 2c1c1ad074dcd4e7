"""MI355X-native hot path of M-AVG (K-step averaging SGD with block momentum).

`kavg` is the binding of the C-ABI library, `configs` the workload table,
`synth` the seeded input generators, `build` compiles the library.
Importing the package loads nothing native; `kavg.load_library()` does.
"""
