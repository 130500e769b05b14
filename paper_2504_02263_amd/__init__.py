"""MI355X-native expert-side MoE hot path: route -> dispatch -> expert FFN -> combine.

`binding` wraps the C ABI of include/moe.h (HIP kernels for gfx950 in csrc/); `roofline`
holds the flop/byte accounting; `build` compiles the shared library.
"""
