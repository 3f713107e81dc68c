"""MI355X-native BLSTM acoustic-model training step with ADPSGD weight mixing.

`inputs` holds the seeded synthetic workloads; `binding` is the thin ctypes layer
over the C-ABI library built from csrc/ (imported on first use, so that the
input generators stay usable on a machine without the built library).
"""
__all__ = ["inputs", "binding", "build"]
