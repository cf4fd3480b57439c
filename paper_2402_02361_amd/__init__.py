"""MI355X-native hot path of Pruner's draft-then-verify schedule exploration (arXiv 2402.02361).

`binding` holds thin wrappers with the names of the C boundary (include/pruner.h):
draft_score, topk, topk_static, prior_filter, lse, random_init, moa_update, verify_score, pacm_score.  They only marshal arguments; every step runs in the HIP
kernels of libpruner_hip.so.  There is no CPU fallback: a missing library raises.
"""
from .binding import (  # noqa: F401
    PrunerError, draft_score, topk, topk_static, prior_filter, lse, random_init, moa_update, time_dominant_draft_launch, verify_score, pacm_score, workspace_bytes, strerror, load_library, library_path,
    NO_COMPUTE_PENALTY, NO_MEMORY_PENALTY, REFERENCE_ROUNDING, FUSED_ARITHMETIC, NSYM, SYMBOL_NAMES, WS_DRAFT, WS_TOPK, WS_VERIFY, WS_PRIOR_FILTER, WS_LSE, WS_PACM,
    CSubgraph, CMlp, CPacm, to_c_subgraphs,
)
