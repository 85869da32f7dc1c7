"""MI355X-native MoE FFN layer with dynamic expert duplication (MoE-GPS setting).

``workloads`` draws seeded synthetic inputs; ``binding`` is the thin ctypes layer
over the C-ABI library ``libmoegps.so`` built from ``csrc/``.
"""
