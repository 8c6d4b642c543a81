"""MI355X-native split feed-forward layer (FFSplit, arXiv 2401.04044).

Thin ctypes binding over libffsplit.so (the C ABI in include/ffsplit.h).  The
binding only marshals arguments; every step of the path runs in the library's
HIP kernels.  PyTorch supplies device memory and the stream, nothing else.
There is no CPU fallback: a missing library raises at import of `binding`.
"""
from .binding import (  # noqa: F401
    ACT_GELU, ACT_SWIGLU, F32, BF16, REM_NONE, REM_DENSE, REM_LOWRANK, REM_INT4, REM_W3H8,
    SCORE_SUMSQ, SCORE_MEAN_L2, SCORE_ACT_ONLY, SCORE_REUSE_TILED,
    WS_SCORE, WS_SELECT, WS_BUILD, WS_FORWARD, WS_FACTORIZE, WS_STACK,
    Desc, FFSplitError, lib, lib_path, status_string, make_desc,
    workspace_bytes, split_bytes, score_neurons, select_heavy, build_split, forward, split_export,
    factorize_remainder, select_heavy_static, SELECT_STATIC_MAX_DFF,
    probe_mfma, probe_stream_read, forward_ex, pack_neuron_bias, token_rmsnorm, stack_forward, Epilogue,
)
