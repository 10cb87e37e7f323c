"""MI355X-native LQ-SGD gradient compressor (HIP kernels behind a C ABI).

`binding` loads the compiled library lazily and raises if it is missing;
`workloads` holds the seeded synthetic inputs.
"""
__all__ = ["binding", "workloads", "build"]
