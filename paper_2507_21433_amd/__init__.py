"""MI355X-native reusable-KV-block search (ReasonCache Sec. IV-A Stage 2 + Sec. IV-B).

``binding`` holds the thin ctypes layer over the C-ABI HIP library; ``synth``
draws the seeded synthetic workloads.  Nothing is loaded at import time.
"""
__version__ = "0.2.0"
