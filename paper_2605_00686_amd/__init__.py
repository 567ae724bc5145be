"""MI355X-native MoE megakernel hot path (route, dispatch, grouped SwiGLU GEMM,
publish with ready flags, combine) behind a C ABI.

`workloads` (seeded synthetic inputs) imports without the HIP library;
`binding` loads `libmoe_hip.so` and raises if it is missing.
"""
