"""MI355X-native KeyDiff block-prefill hot path (hand-written HIP for gfx950).

The product is ``libkeydiff.so`` (C ABI in ``include/keydiff.h``); this package
is the thin ctypes binding over it.  There is no CPU fallback: importing
``binding`` without the built library raises.
"""
from .binding import (  # noqa: F401
    ANCHOR_MEAN_KEY,
    ANCHOR_MEAN_UNIT_KEY,
    KERNEL_NAMES,
    LAYOUT_FILL,
    LAYOUT_ORDERED,
    KeyDiffCache,
    KeyDiffConfig,
    KeyDiffError,
    load_library,
    prefill_block_layers,
)
