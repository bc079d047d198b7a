"""MI355X-native alternating-least-squares hot path (hand-written HIP for gfx950 behind a C ABI)."""
from .binding import (Als, AlsError, SparseMatrix, load_library, SOLVER_CHOLESKY, SOLVER_CG,  # noqa: F401
                      K_HERMITIAN, K_SOLVE, K_RMSE, K_PLAN, K_FUSED, K_GRAM, K_SHORT, EXPORTS, F32, BF16, F16, F32X3, F32X2,
                      PEAK_MFMA_F32, PEAK_MFMA_BF16, PEAK_MFMA_F16, PEAK_COPY,
                      ALS_OK, ALS_EINVAL, ALS_EHIP, ALS_ENUMERIC, ALS_ENOMEM)
