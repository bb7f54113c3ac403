"""MI355X-native Kernel-SHAP edge attribution for GCNs (DistShap hot path).

The computation lives in `libdistshap_hip.so` (hand-written HIP for gfx950,
C ABI declared in include/distshap.h). This package is only the ctypes
marshalling layer around it; PyTorch supplies device memory and streams.
"""
from .binding import (DistShapError, Context, Options, Report, Tuning, CGraphInfo, load_library,
                      library_path, DS_OK, DS_EINVAL, DS_ECAPACITY, DS_ENOMEM, DS_ENOTCONV,
                      DS_EDEVICE, DS_ESINGULAR, DS_EINTERNAL, DS_F32, DS_BF16_IN_F32_ACC,
                      DS_SCORE_PROB, DS_SCORE_LOGIT, DS_SOLVER_AUTO, DS_SOLVER_GRAM_CHOL,
                      DS_SOLVER_CGLS, EXPORTED_SYMBOLS)
