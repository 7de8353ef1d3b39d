"""MI355X-native speculative decoding rounds for patch-autoregressive time-series transformers.

The product is the C-ABI library `libtsd.so` (declared in include/tsd.h, implemented as HIP
kernels for gfx950).  This package is its thin Python binding: argument marshalling only.
"""
from .binding import (  # noqa: F401
    TSD_BF16, TSD_DRAFT, TSD_F32, TSD_FLAG_NAIVE_VERIFY, TSD_FLAG_NO_COMPACT, TSD_FLAG_NO_GRAPH, TSD_FLAG_NO_SKINNY, TSD_FLAG_NO_TEMPERING,
    TSD_FLAG_SAMPLE_PROPOSALS, TSD_FLAG_SCRAMBLE_PAGES, TSD_FLAG_THRESHOLD_RULE, TSD_FLAG_BATCH_SYNC, TSD_FLAG_NO_PINNED_COUNTS, TSD_FLAG_NO_FUSED_DRAFT, TSD_FLAG_FUSED_DRAFT, TSD_FLAG_NO_WIDE_GEMM, TSD_TARGET, TsdConfig, TsdError,
    TsdModelCfg, TsdStats, Session, accept_commit_static, bench_copy, bench_gemm, bench_mfma, lib, library_path, make_config, session_for,
)
from . import law  # noqa: F401,E402
