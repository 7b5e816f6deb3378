"""MI355X-native hot path of NOVA's entropy-guided token reduction.

The product is the C-ABI library built from ``csrc/`` (see ``include/nova.h``);
this package is its thin Python binding.  There is no CPU fallback: importing
:mod:`paper_2602_01345_amd.binding` works anywhere, but creating a
:class:`~paper_2602_01345_amd.binding.Nova` handle raises if ``libnova.so`` is
not built or no GPU is present.
"""
from .binding import (NOVA_BF16, NOVA_F32, BlockShape, BlockVariant, Nova, NovaError, activation_scale, library_path,
                      load_library, pack_k_cache, pack_v_cache, scale_ratio, unpack_k_rows, unpack_v_rows)

__all__ = ["Nova", "NovaError", "BlockShape", "BlockVariant", "NOVA_F32", "NOVA_BF16", "load_library", "library_path",
           "pack_k_cache", "pack_v_cache", "unpack_k_rows", "unpack_v_rows", "activation_scale", "scale_ratio"]
