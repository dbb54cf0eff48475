"""libseedinf: SEED RL's central batched inference step, hand-written HIP for gfx950.

`workloads` holds the seeded synthetic input generators; `seedinf` is the thin
ctypes binding over the C-ABI library built from `csrc/`.
"""
__all__ = ["workloads", "seedinf"]
