"""MI355X (gfx950) LASER routing step behind a C ABI (include/laser.h).

`paper_2510_03293_amd.binding` is the ctypes front end; `build` compiles the HIP
sources in `csrc/` into `liblaser_route.so` next to this file.
"""
