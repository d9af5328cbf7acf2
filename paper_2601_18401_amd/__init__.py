"""MI355X-native span-search / span-attention (N = 2 Superlinear attention hot path).

`paper_2601_18401_amd.binding` is the thin ctypes layer over the C-ABI library libsl.so
(hand-written HIP for gfx950); `paper_2601_18401_amd.workloads` holds the seeded synthetic
input generators; `paper_2601_18401_amd.build` compiles the library in-tree.
"""
