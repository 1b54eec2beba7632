"""MI355X-native RTN ternary conv/GEMM hot path (HIP kernels behind a C ABI).

`binding` loads the HIP library on first use and raises if it is missing;
`workloads` only draws seeded synthetic inputs.
"""
