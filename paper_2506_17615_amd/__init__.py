"""MI355X-native block-wise int8 quantized P-way reduction (the compute path of EQuARX).

``binding`` wraps the C-ABI library built from ``csrc/``; ``workloads`` holds the
seeded synthetic input recipes.  Importing the package loads nothing native:
the HIP library is opened on first use of ``binding`` and its absence is an error.
"""
__all__ = ["binding", "workloads", "build"]
