"""MI355X-native forward of a fully quantized linear layer with a quantized low-rank branch.

``paper_2604_18117_amd.binding`` is the thin ctypes layer over the C-ABI library built from
``csrc/``; ``paper_2604_18117_amd.workloads`` holds layer shapes and seeded input generators.
Importing this package loads nothing; importing ``binding`` fails loudly if the HIP library
has not been built.
"""
