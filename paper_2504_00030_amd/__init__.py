"""MI355X-native speculative-decoding step (draft decode, target verification, accept / resample)
with the GammaTune speculation-length controller.  See include/spec.h and include/gammatune.h."""
from .binding import (  # noqa: F401
    ACCEPT_FORCED, ACCEPT_NATURAL, GT_EXPAND_A, GT_LITERAL, GT_SHORT_TERM, PATH_AUTO, PATH_MFMA, PATH_WAVEDOT,
    FixedGamma, GammaTune, SpecEngine, SpecError, k_accept, k_accept_static, k_copy, k_gemm_tiled, k_gemm_tiled_q8, k_gemv, k_gemv_tiled, k_gemv_tiled_q8, k_philox, k_retile, k_retile_q8, load,
)
