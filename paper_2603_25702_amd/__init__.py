"""MI355X-native S2D2 draft + verify + accept + cache-append step (hand-written HIP, C ABI).

`binding` marshals torch device tensors into the C ABI of libs2d2.so (include/s2d2.h); every
step of the path runs in the library's kernels.  Nothing here falls back to the CPU: loading
fails loudly if the library has not been built (python -m paper_2603_25702_amd.build).
"""
from .binding import (  # noqa: F401
    AcceptOut, BlockState, DraftOut, Engine, KvCache, Params, S2D2Error, VerifyOut, lib_path, load_library,
)
