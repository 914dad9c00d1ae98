"""MI355X-native out-of-core CNN training step (keep / swap / recompute per feature map).

The product is libpooch.so (HIP, gfx950) behind the C ABI of include/pooch.h; this package
holds its sources (csrc/), the build step (build.py) and a ctypes binding (binding.py).
"""
from .binding import (BudgetError, Context, PoochError, KEEP, SWAP, RECOMPUTE, MODES, SYMBOLS, lib)  # noqa: F401
