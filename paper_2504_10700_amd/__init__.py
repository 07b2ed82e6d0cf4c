"""MI355X-native MACE symmetric tensor contraction (forward, dA, dW).

`workloads` holds the seeded synthetic input recipes; `binding` is the thin
ctypes layer over the C-ABI library built from `csrc/` (imported on first use,
so that importing the package never needs the built library).
"""
__all__ = ["workloads", "binding"]
