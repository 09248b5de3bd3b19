"""MI355X-native stacked-LSTM forward/BPTT library (HIP kernels behind a C ABI).

`binding` forwards to the compiled library; `inputs` draws the seeded synthetic
workloads; `build` compiles the library in-tree.  Nothing is loaded at import.
"""
