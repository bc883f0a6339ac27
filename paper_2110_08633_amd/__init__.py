"""MI355X-native spilled, shard-alternated multi-model decoder training.

Thin ctypes binding over libhydra.so (hand-written gfx950 HIP kernels behind a
C ABI).  Every step of the path runs in the library; Python only marshals
arguments and uses torch for device memory, pinned memory and streams.
"""
from . import hydra  # noqa: F401
