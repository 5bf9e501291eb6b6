"""SBO dictionary-learning iteration on MI355X: ctypes binding of libsbo (HIP, gfx950)."""
from .binding import (EXPORTS, SBO_OPT_SVD_METHOD, SBO_OPT_CODING_ARITH, SBO_SVD_AUTO, SBO_SVD_JACOBI, SBO_ARITH_F32, SBO_ARITH_BF16X3, SBO_ARITH_BF16X3_SCREEN, SBO_ARITH_F16X2, LIB_PATH, STAGES, SboError, lib, sbo_accumulate, sbo_code,  # noqa: F401
                      sbo_create, sbo_destroy, sbo_group, sbo_group_static, sbo_init_base, sbo_iterate, sbo_learn, sbo_new_base, sbo_set_blocks,
                      sbo_polar, sbo_set_option, sbo_set_timing, sbo_sqerr, sbo_stage_ms, sbo_strerror, sbo_svd_sweeps,
                      sbo_train_rounds, sbo_update, sbo_workspace_bytes, sbo_worst)
