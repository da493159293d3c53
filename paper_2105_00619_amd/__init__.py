"""MI355X-native sequential-checkpoint training step (gradient-flow optimisation of OpTorch).

`workloads` describes networks and draws seeded inputs; `binding` is the thin
ctypes layer over the C-ABI library built from `csrc/`.  The binding is loaded
lazily so that the input generators can be used without the GPU library.
"""

__all__ = ["workloads", "binding"]
