"""MI355X-native block-span inference server path (C ABI in include/span.h).

The Python layer only marshals arguments into libspan.so; every step of the path runs
in the HIP kernels.  There is no CPU fallback: if the library is missing, importing
`paper_2312_08361_amd.binding` raises.
"""
