"""MI355X-native V-step re-encoding for PV-Tuning (arXiv 2405.14852).

The product is the C-ABI library libpv.so (include/pv.h, sources in csrc/).
This package is its thin Python binding: argument marshalling only.
"""
from .binding import (PVContext, PVError, Layout, KERNEL_IDS, library_path, load_library)

__all__ = ["PVContext", "PVError", "Layout", "KERNEL_IDS", "library_path", "load_library"]
