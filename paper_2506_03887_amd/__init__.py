"""MI355X-native batched token-mask path of Pre^3 (arXiv 2506.03887).

The product is libpre3.so (csrc/: HIP kernels for gfx950 behind the C ABI of include/pre3.h);
`binding` marshals torch tensors into it.
"""
from .binding import Pre3, Pre3Error, apply_mask, load  # noqa: F401
