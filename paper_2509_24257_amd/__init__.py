"""MI355X-native verification hot path (teacher-forced prefill + compare) behind a C ABI.

`paper_2509_24257_amd.binding` is a thin ctypes layer over libverillm.so with the same function names
as include/verillm.h; every step of the path runs inside that library's HIP kernels.
"""
from .binding import (  # noqa: F401
    VL_BF16, VL_F32, VerilLMError, Context, ModelCfg, Summary, Tol, TokStats, BitRule, BitStats, lib, lib_path, load_library,
    vl_plan_memory,
)
