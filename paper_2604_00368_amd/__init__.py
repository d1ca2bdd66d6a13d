"""MI355X-native slice split / rail binding / gather-scatter engine (TENT data-plane hot path).

``workloads`` builds seeded synthetic inputs; ``binding`` is the thin ctypes
layer over the C-ABI library built from ``csrc/``.
"""
