"""MI355X-native GPU embedding cache (level-1 store of the Hierarchical Parameter Server).

`inputs` holds the seeded synthetic generators; `binding` is the thin ctypes layer over the
C-ABI library built from `csrc/`.  Nothing here falls back to a CPU implementation: using the
cache without the built HIP library raises.
"""
