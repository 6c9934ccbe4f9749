"""MI355X-native Block Transformer generation step (arXiv 2406.02657).

The product is the C-ABI library libbt.so (hand-written gfx950 HIP kernels);
this package is a thin ctypes binding with the same entry-point names.  There
is no CPU fallback: importing `binding` without a built library raises.
"""
from .binding import (  # noqa: F401
    BT_F32, BT_BF16, BTError, Model, bt_config, bt_layer_weights, bt_stats, bt_weights, lib, lib_path,
)
