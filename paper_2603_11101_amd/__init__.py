"""Packed variable-length attention for MI355X (gfx950): host packer, C-ABI
library of hand-written HIP kernels, and a thin ctypes binding.

``workloads`` (seeded synthetic inputs) imports nothing else; ``binding``
loads the built shared library and fails loudly when it is missing.
"""
