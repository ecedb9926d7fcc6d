"""MI355X-native integer-only ViT encoder forward (I-ViT, arXiv 2207.01405).

`paper_2207_01405_amd.binding` is the thin ctypes layer over the C-ABI library
(libivit.so, hand-written HIP for gfx950); `paper_2207_01405_amd.synth` draws the
seeded synthetic workloads.  There is no CPU fallback: every call into the binding
raises if the HIP library has not been built.
"""
