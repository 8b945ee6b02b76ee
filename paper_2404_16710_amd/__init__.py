"""MI355X-native greedy self-speculative decoding (early-exit drafts, remaining-layer verify).

The work is done by hand-written HIP kernels behind the C ABI in include/ls.h
(libls.so, built in-tree by `paper_2404_16710_amd.build`).  This package only marshals
arguments: torch provides device memory and streams, nothing else.
"""
from .binding import (  # noqa: F401
    LsError, LsModel, Stats, DeviceWeights, generate_static, lib, lib_path, config_struct, LS_F32, LS_BF16,
)
