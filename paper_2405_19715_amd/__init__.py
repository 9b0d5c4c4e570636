"""MI355X-native draft-verify-correct round of speculative decoding with adaptive
candidate length (SpecDec++, Algorithm 2): hand-written HIP kernels for gfx950
behind a C-ABI library, plus a thin ctypes binding with the same names.

`synth` (seeded synthetic inputs) imports without the library; everything in
`binding` needs the built `libspecdec.so` and raises if it is missing.
"""
