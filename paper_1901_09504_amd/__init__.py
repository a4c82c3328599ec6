"""OCS-expanded quantized layer for AMD MI355X: hand-written HIP behind a small C ABI.

`binding` holds the ctypes front end of libocs.so, `build` compiles it, `workloads` draws
the seeded synthetic layers.  Nothing is loaded at import time.
"""
