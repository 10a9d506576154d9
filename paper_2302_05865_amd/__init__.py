"""Flag Aggregator hot path for AMD MI355X: thin Python binding over the C ABI in
``include/fa.h`` (``libfa.so``, hand-written HIP kernels).  Argument marshalling only --
every step of the path runs in the library's kernels.  PyTorch is used by callers for device
memory and streams; this package only needs raw device addresses.
"""
from ._binding import (FlagAggregator, FaError, FaInfoResult, fa_aggregate_static, library_path,
                       load_library, EXPORTED_SYMBOLS)

__all__ = ["FlagAggregator", "FaError", "FaInfoResult", "fa_aggregate_static", "library_path",
           "load_library", "EXPORTED_SYMBOLS"]
