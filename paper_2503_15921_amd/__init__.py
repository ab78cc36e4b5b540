"""Python binding of libspin: the batched verification step of speculative decoding on MI355X.

Argument marshalling only -- every step (scheduling, attention, acceptance) runs inside the
C-ABI library built from csrc/.  PyTorch is used for device memory and streams.  There is no
CPU fallback: if libspin.so is missing, importing the entry points raises.
"""
from .binding import (  # noqa: F401
    SpinError, SpinContext, accept_noalloc, decompose, kv_padding, check_tiling, schedule, lib_path, load_library,
    DECOMP_NONE, DECOMP_Q_SPLIT, DECOMP_KV_SPLIT, DECOMP_KV_SEARCH, ACCEPT_GREEDY, ACCEPT_REJECTION,
    EINVAL, ETABLE, ENOSPC, EUNSUPPORTED, EHIP, PIECE_CARRY_IN, PIECE_CARRY_OUT, PIECE_DIRECT, PIECE_QUEUED,
)
