"""MI355X-native adapter cache pool + batched heterogeneous-rank LoRA apply.

The product is liblora_cache.so (C ABI in include/lora_cache.h, HIP kernels for gfx950 in
csrc/).  This package is the thin Python face over it: `binding` mirrors the C calls one to
one, `pool` adds the few lines that get device memory and streams from PyTorch.
"""
from . import binding  # noqa: F401  (raises ImportError if the library is not built)
from .binding import *  # noqa: F401,F403
from .pool import LoraPool  # noqa: F401
