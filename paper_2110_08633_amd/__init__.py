"""MI355X-native spilled, shard-alternated multi-model decoder training.

Thin ctypes binding over libhydra.so (hand-written gfx950 HIP kernels behind a
C ABI).  Every step of the path runs in the library; Python only marshals
arguments and uses torch for device memory, pinned memory and streams.
"""
# The binding (`paper_2110_08633_amd.hydra`) loads libhydra.so at import and fails loudly when the library is missing
# or stale; it is not imported here so that `paper_2110_08633_amd.build` can run on a tree without the library.
