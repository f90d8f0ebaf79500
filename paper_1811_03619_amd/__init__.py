"""MI355X-native Pipe-SGD aggregation + update path (arXiv 1811.03619).

The compute lives in ``csrc/`` (HIP kernels behind a C ABI, built into
``libpipesgd.so``); ``binding`` marshals arguments to it; ``workloads`` holds
seeded synthetic inputs.  Nothing is loaded at import time: the library is
opened on first use and every call raises if it is missing.
"""
__all__ = ["binding", "workloads", "buildlib"]
