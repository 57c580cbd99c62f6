"""MI355X-native MOSS FP8 hot path: thin Python binding over the C-ABI HIP library.

Importing the package loads nothing; the first call of a binding function loads
paper_2511_05811_amd/libmoss_hip.so and fails loudly if it has not been built
(`python -m paper_2511_05811_amd.build`).  There is no CPU fallback.
"""
from .binding import (  # noqa: F401
    MOSS_DT_BF16, MOSS_DT_F32, MOSS_EXP_CEIL, MOSS_EXP_NEAREST, MOSS_Q_COL, MOSS_Q_ROW, MOSS_WS_KEPT, MOSS_WSTATE_STEP_MISMATCH,
    AdamWArgs, MossError, WScaleState, device_cu_count, exported_symbols, gemm_bf16_baseline,
    gemm_fp8_mx, lib_path, load, quant_act_2level, quant_act_2level_given_max, quant_act_2level_noalloc, quant_set_poll_limit, read_wscale_state, weight_autoscale_cast,
    weight_autoscale_init, new_wscale_state, swiglu_bf16, swiglu_bf16_backward, add_rmsnorm_bf16, rmsnorm_bf16_backward,
)
