"""MI355X-native ROCKET random-convolutional-kernel transform (gfx950, HIP).

`synth` holds the seeded workload generators; the C-ABI binding lives in
`paper_2301_08527_amd.rocket` and is imported lazily so that the generators
can be used without the native library.
"""
