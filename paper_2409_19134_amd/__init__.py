"""SPD decode-attention hot path for AMD MI355X: HIP library + ctypes binding (see include/spd.h)."""
from .binding import (Context, KVView, SpdError, make_shape, spd_build_schedule, spd_strerror,  # noqa: F401
                      spd_validate_partial, spd_kv_view, spd_shape, spd_work_item, lib, LIB_PATH,
                      EXPORTED_SYMBOLS, SPD_OK, SPD_ERR_NULL, SPD_ERR_SHAPE, SPD_ERR_LEN, SPD_ERR_ALIGN,
                      SPD_ERR_WORKSPACE, SPD_ERR_HIP, SPD_ERR_NOMEM, SPD_F32, SPD_BF16, SPD_F16, SPD_OPT_HEAD_PER_WAVE, SPD_OPT_TARGET_WG_PER_CU,
                      SPD_OPT_NO_SPLIT_MAX, SPD_OPT_CHUNK_MAX, SPD_OPT_SEG_COST, SPD_OPT_HALF_SKEW,
                      SPD_OPT_RESULT_ROWS, SPD_OPT_STEPS_IN_FLIGHT)
from .step import DecodeStep  # noqa: F401,E402
