"""MI355X (gfx950) Sparse Window Attention decode path behind a C ABI.

`binding` holds the ctypes front end of libswa_hip.so (same names as the C entry
points), `workload` the seeded synthetic inputs, `build` the hipcc build step.
"""
