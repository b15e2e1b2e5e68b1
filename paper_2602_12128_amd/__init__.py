"""MI355X-native Hadamard Linear Attention: thin Python binding over the C-ABI library libhla.so.

Importing this package does not load the library; the first use of the binding does, and fails
loudly if libhla.so has not been built (there is no CPU fallback)."""
from .binding import (HLA, hla_forward_static, HLAError, HLA_BF16, HLA_F32, HLA_OK, HLA_PATH_AUTO, HLA_PATH_GENERIC,
                      HLA_PATH_MFMA, HLA_PHI_MLP, HLA_PHI_NONE, load_library, status_string)

__all__ = ["HLA", "hla_forward_static", "HLAError", "HLA_BF16", "HLA_F32", "HLA_OK", "HLA_PATH_AUTO", "HLA_PATH_GENERIC",
           "HLA_PATH_MFMA", "HLA_PHI_MLP", "HLA_PHI_NONE", "load_library", "status_string"]
