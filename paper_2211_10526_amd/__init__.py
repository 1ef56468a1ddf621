"""MI355X-native linear-angular attention (inference path of Castling-ViT).

csrc/      HIP kernels and the C ABI (include/castling_attn.h)
binding    ctypes binding with the same entry points
inputs     seeded synthetic workloads
build      hipcc driver for libcastling_attn.so
"""
