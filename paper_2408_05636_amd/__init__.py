"""MI355X (gfx950) implementation of one Speculative Diffusion Decoding round (arxiv 2408.05636).

`synth` holds the seeded input generators, `binding` the ctypes layer over libspecdiff.so
(hand-written HIP kernels behind a C ABI, see include/specdiff.h), `build` compiles it.
"""
