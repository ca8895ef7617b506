"""MI355X-native ROCKET random-convolutional-kernel transform (gfx950, HIP).

The C-ABI binding lives in
`paper_2301_08527_amd.rocket`; `build.py` compiles the library in-tree.
"""
