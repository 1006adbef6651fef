"""MI355X-native relay-race ranking path (prefix pre-inference, ranking on cached prefix K/V,
full recompute, HBM K/V pool) behind the C ABI of include/relaygr.h.

`binding` marshals arguments into librelaygr.so; every step of the path runs in the HIP
kernels under csrc/.  There is no CPU or PyTorch fallback: without the built library (and,
for compute calls, a GPU) the calls fail.
"""
from .binding import *  # noqa: F401,F403
from .binding import (  # noqa: F401
    Batch, Context, KvPool, RelayGRError, EXPORTS, load_library, make_config,
)
