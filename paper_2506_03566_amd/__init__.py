"""MI355X-native PosS draft-and-verify round: thin Python binding of libposs.so.

All computation happens in the HIP library (csrc/); importing this package
without a built libposs.so works, using it raises.
"""
from .binding import (Poss, PossError, PossConfig, PossTree, PossStats, TreeArrays, load_library,  # noqa: F401
                      make_config, debug_gemm, gemm_static, GEMM_STATIC_BYTES, EXPORTS, LIB_PATH, MAX_ROWS, MASK_WORDS, MAX_DEPTH,
                      POSS_OK, E_INVALID_ARG, E_BAD_STATE, E_CAPACITY, E_BAD_TREE, E_HIP)
