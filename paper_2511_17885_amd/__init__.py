"""MI355X-native MoE-layer prefill path of FastMMoE (modality-dependent top-k routing,
routing-aware visual-token pruning, expert grouped GEMM, gate-weighted combine).

The compute lives in a C-ABI HIP library (`csrc/`, declared in `include/fmoe.h`);
`binding` is a thin ctypes layer over it and `workloads` draws seeded synthetic inputs.
Importing the package does not load the library; the first call into `binding` does and
raises if it has not been built.
"""
__all__ = ["workloads", "binding"]
