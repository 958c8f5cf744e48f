"""MI355X-native HiViS draft-verify decode path: HIP kernels behind a C ABI (csrc/, include/hivis.h)
and a thin ctypes binding.  Importing this package loads nothing; `Hivis(...)` loads libhivis.so."""
from .binding import (Hivis, HivisError, load_library, calib_stream, EXPORTED_SYMBOLS, LIB_PATH, HIVIS_OK, HIVIS_EINVAL,
                      HIVIS_ESTATE, HIVIS_ECAP, HIVIS_EHIP, HIVIS_F32, HIVIS_BF16)

__all__ = ["Hivis", "HivisError", "load_library", "calib_stream", "EXPORTED_SYMBOLS", "LIB_PATH"]
