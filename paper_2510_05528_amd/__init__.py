"""MI355X-native ARMOR per-layer factorization: thin Python binding over the C ABI (include/armor.h).

Only argument marshalling happens here; every step of the path runs in the HIP kernels of
libarmor.so.  torch is used for device memory and streams.  There is no CPU fallback: if the
library is missing, every call raises.
"""
from .binding import (ARMOR_BF16, ARMOR_F32, ArmorError, apply_packed, apply_prepare, apply_workspace_bytes, to_bf16, factorize_layer, factorize_workspace_bytes, gram,
                      gram_diag, gram_diag_x, gram_workspace_bytes, load_library, normalize, pack_mask, pack_nm, profile_enable, profile_read, proxy_loss, proxy_loss_full_h, proxy_loss_noalloc, unpack_mask, unpack_meta)

__all__ = ["ARMOR_BF16", "ARMOR_F32", "ArmorError", "apply_packed", "apply_prepare", "apply_workspace_bytes", "to_bf16", "factorize_layer", "factorize_workspace_bytes", "gram",
           "gram_diag", "gram_diag_x", "gram_workspace_bytes", "load_library", "normalize", "pack_mask", "pack_nm", "profile_enable", "profile_read", "proxy_loss", "proxy_loss_full_h", "proxy_loss_noalloc",
           "unpack_mask", "unpack_meta"]
