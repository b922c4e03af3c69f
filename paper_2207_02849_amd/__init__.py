"""MI355X-native hypergradient kernels (Neumann / finite-difference implicit differentiation).

`binding` wraps the C-ABI library; `workloads` draws the seeded synthetic inputs;
`build` compiles the HIP sources.  Importing the package loads nothing.
"""
