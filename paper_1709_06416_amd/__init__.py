"""weld-hip: the fused data-parallel `for` loop of Weld, native on MI355X (gfx950).

`binding` wraps the C ABI of libweldhip.so (include/weld_hip.h); `build` compiles it.
"""
