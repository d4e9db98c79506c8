"""MI355X-native NSA speculative-verification attention (the hot path of SSV, arxiv 2605.19893).

The product is the HIP library behind include/ssv_nsa.h; this package is its thin Python binding.
"""
from .binding import (SSV_BF16, SSV_F32, SSV_REFRESH, SSV_REFRESH_SHARED, SSV_REUSE, SsvCmpParams, SsvError, SsvNsaParams, SsvNsaPlan,  # noqa: F401
                      load_library, make_cmp_params, make_params, ssv_nsa_compress, ssv_nsa_plan_query, ssv_nsa_supported, ssv_nsa_verify,
                      ssv_nsa_verify_static, ssv_nsa_workspace_bytes)
