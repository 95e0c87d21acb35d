"""Python binding of libltri (argument marshalling only; every step runs in the HIP kernels)."""
from .binding import (LtriConfig, LtriContext, LtriError, config_from_workload, load_library,
                      library_path, EXPORTED_SYMBOLS)

__all__ = ["LtriConfig", "LtriContext", "LtriError", "config_from_workload", "load_library",
           "library_path", "EXPORTED_SYMBOLS"]
