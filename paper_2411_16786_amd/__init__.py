"""MI355X-native MoE expert layer with DICE conditional refresh (gfx950, HIP).

``paper_2411_16786_amd.binding`` is the thin ctypes layer over the C-ABI library
``libdicemoe.so`` (built from ``csrc/``); ``paper_2411_16786_amd.workloads`` holds
the seeded synthetic inputs.  Nothing is loaded at import time: the binding
loads the library on first use and raises if it is missing.
"""
__all__ = ["binding", "workloads", "build"]
