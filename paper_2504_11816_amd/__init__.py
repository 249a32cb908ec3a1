"""Decode attention over a partly offloaded KV cache for one MI355X.

binding   ctypes layer over libokv.so (the C ABI declared in include/okv.h)
harness   device / pinned-host buffers and streams around a binding.Context
synth     seeded synthetic inputs (shared with the tests' CPU oracle)
build     hipcc driver that produces libokv.so next to this file
"""
