"""MI355X-native hot path of MSched's proactive memory scheduling (arXiv 2512.24637):
plan a migration at each context switch and carry it out, as HIP kernels behind the
C ABI declared in include/msched.h.  This package is the thin Python binding."""
from .binding import (MSched, MSchedError, Plan, load_library, library_path, NOT_RESIDENT,
                      EXPORTED_SYMBOLS, PHASES, analyze, rules_from_bytes)

__all__ = ["MSched", "MSchedError", "Plan", "load_library", "library_path", "NOT_RESIDENT",
           "EXPORTED_SYMBOLS", "PHASES", "analyze", "rules_from_bytes"]
