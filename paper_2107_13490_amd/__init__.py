"""MI355X-native fixed-point hot path of AdaPT (arXiv 2107.13490).

Thin ctypes binding over the C ABI declared in include/adapt_fxp.h.  Every step of the path
runs in the HIP library (paper_2107_13490_amd/libadapt_fxp.so); PyTorch only provides device
memory and streams.  There is no CPU fallback: if the library is missing, loading raises.
"""
from .binding import (  # noqa: F401
    CALL_CONV_BACKWARD, CALL_CONV_DGRAD, CALL_CONV_FWD, CALL_CONV_WGRAD, CALL_GEMM, CALL_GRADIENT_DIVERSITY, CALL_KLD_SEARCH,
    CALL_KLD_SEARCH_BATCHED, CALL_QUANTIZE, CALL_QUANTIZE_BATCHED, CALL_REQUANTIZE_FIT, CALL_SGD_UPDATE, WorkspaceQuery,
    NT_A, NT_BN, NT_DA, NT_DBETA, NT_DGAMMA, NT_DY, NT_DYC, NT_EXP, NT_G, NT_INPUT, NT_QW, NT_STATS, NT_Y, NT_YC, NodeDesc, RN_HALF_UP, SR, ST_MAX, ST_MEAN, ST_MIN, AdaptError, Context,
    ConvDesc, Epilogue, Fmt, LayerDesc, Net, NetStats, Rng, SwitchParams, SwitchReport, acc_bits,
    library_path, load_library, lookback_next, perf_model_size, perf_step_cost, perf_step_memory, perf_step_overhead,
    pushup_suggest, resolution_next, strategy_next,
)
