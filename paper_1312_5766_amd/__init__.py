"""MI355X-native hot path of SAP/STRADS-scheduled Lasso coordinate descent.

The product is libstrads_lasso.so (hand-written HIP for gfx950, C ABI in
include/strads_lasso.h); this package is its thin Python binding."""
from .binding import (StradsLasso, StradsError, RoundInfo, RunInfo, load, LIB_PATH, EXPORTS,  # noqa: F401
                      strads_lasso_workspace_bytes, LAYOUT_DENSE, LAYOUT_CSC, LAYOUT_GENO2, MAX_L_PRIME,
                      DEPS_STATIC, DEPS_DYNAMIC, DEPS_NONE, PRIORITY, STAGE_NAMES, STRADS_OK, E_INVALID_ARG,
                      E_WORKSPACE_TOO_SMALL, E_HIP, E_DIVERGED, E_UNSUPPORTED, E_TOO_LARGE, FILTER_STATIC_MAX_L,
                      strads_lasso_filter_static, strads_lasso_gram256_plan,
                      strads_lasso_gram_default_tile_edge)
