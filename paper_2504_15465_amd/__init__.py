"""MI355X-native kernel atomization and CU-partition scheduling (LithOS hot path).

``inputs`` draws seeded synthetic workloads; ``binding`` is the thin ctypes
layer over the C-ABI library ``liblithos.so`` (loaded lazily, on first use).
"""
__all__ = ["inputs", "binding"]
