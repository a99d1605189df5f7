"""KVComp hot path for MI355X (gfx950): hand-written HIP kernels behind the C ABI of include/kvcomp.h.

`binding` holds the ctypes layer (needs torch and the built libkvcomp.so); `build` compiles the library.
Nothing is loaded at import time.
"""
