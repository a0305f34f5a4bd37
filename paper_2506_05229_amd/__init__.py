"""MI355X-native Diagonal Batching forward pass of an ARMT (arxiv 2506.05229).

The product is the C-ABI shared library built from csrc/ (declared in include/armt.h);
`binding` is a thin ctypes layer over it that marshals torch device tensors."""
from .binding import (ArmtConfig, ArmtLayerWeights, ArmtLayerGrads, Armt, load_library, library_path, ArmtError,
                      diagonal_group, grouped_gemm, ArmtSteps, set_gemm_tile_config, profile_begin,
                      profile_end, GEMM_KINDS, TokenEnds)

__all__ = ["ArmtConfig", "ArmtLayerWeights", "ArmtLayerGrads", "Armt", "load_library", "library_path", "ArmtError",
           "diagonal_group", "grouped_gemm", "ArmtSteps", "set_gemm_tile_config", "profile_begin", "profile_end", "GEMM_KINDS",
           "TokenEnds"]
