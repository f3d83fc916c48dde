"""libq4kv for AMD MI355X: batched attention over paged 4-bit KV caches and the Q4 codec.

`binding` holds the entry points (same names as include/q4kv.h); `synth` draws the seeded
benchmark inputs.  Importing this package does not load the shared library; the first call does,
and raises if it has not been built.
"""
