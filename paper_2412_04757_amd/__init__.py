"""Python binding of libltri (argument marshalling only; every step runs in the HIP kernels)."""
from .binding import (LtriConfig, LtriContext, LtriError, config_from_workload, load_library,
                      library_path, EXPORTED_SYMBOLS, measure_mfma_peak, measure_copy_peak, measure_read_peak,
                      REP_MEAN, REP_DYNAMIC, RATIO_ROW, RATIO_COL, RATIO_ROWCOL)

__all__ = ["LtriConfig", "LtriContext", "LtriError", "config_from_workload", "load_library",
           "library_path", "EXPORTED_SYMBOLS", "measure_mfma_peak", "measure_copy_peak", "measure_read_peak",
           "REP_MEAN", "REP_DYNAMIC", "RATIO_ROW", "RATIO_COL", "RATIO_ROWCOL"]
