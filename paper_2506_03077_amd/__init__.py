"""StreamBP hot path for MI355X (gfx950): ctypes binding over libstreambp.so.

`binding` mirrors the C ABI declared in include/streambp.h; `synth` draws the
seeded synthetic inputs; `build` compiles the library in-tree.
"""
