"""MI355X-native cacheless MoE decode layer (OD-MoE hot path).

`synth` makes seeded inputs; `binding` is the ctypes layer over libodmoe.so
(loaded on first use; importing this package never touches the GPU).
"""
__all__ = ["synth", "binding"]
