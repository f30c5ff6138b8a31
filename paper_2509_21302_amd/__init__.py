"""qvggt: W4A4 Dual-Smoothed Fine-Grained Quantization linear layer for MI355X (gfx950).

The product is the C-ABI shared library libqvggt.so (declared in include/qvggt.h, built from
csrc/ by build.py); `binding` is the thin ctypes layer with the same entry-point names.
"""
from . import binding as _binding
from .binding import QvggtError, lib_path, load_library, EXPORTS, QVGGT_BF16, QVGGT_F32  # noqa: F401

# every entry point of the C ABI under its own name (binding.EXPORTS lists them; tests check the list against include/qvggt.h)
for _name in EXPORTS:
    globals()[_name] = getattr(_binding, _name)
del _name

from .module import DsfqLinear  # noqa: E402,F401
