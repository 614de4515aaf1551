"""MI355X executor for synthesized operators: thin Python face of the C ABI in include/syno.h.

Importing this package does not load the HIP library; `binding` does, on first use, and
raises if it has not been built (`python -m paper_2410_23745_amd.build`).
"""
from .binding import BWD_DATA, BWD_WEIGHT, FWD, Chain, Plan, SynoError, library_path, load_library, mfma_rate

__all__ = ["Plan", "Chain", "SynoError", "FWD", "BWD_DATA", "BWD_WEIGHT", "library_path", "load_library", "mfma_rate"]
