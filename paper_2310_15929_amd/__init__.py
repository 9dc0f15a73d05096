"""MI355X-native E-Sparse hot path: thin ctypes binding over libesparse.so (gfx950)."""
from .binding import (Context, PruneOpts, PruneResult, Compressed, EsparseError, load_library,
                      compressed_size, spmm_workspace, dense_packed_size, num_variants, variant_name,
                      F16, BF16, USE_ENTROPY, USE_NORM, USE_GNS, USE_LBS, USE_ALL)

__all__ = ["Context", "PruneOpts", "PruneResult", "Compressed", "EsparseError", "load_library",
           "compressed_size", "spmm_workspace", "dense_packed_size", "num_variants", "variant_name",
           "F16", "BF16", "USE_ENTROPY", "USE_NORM", "USE_GNS", "USE_LBS", "USE_ALL"]
