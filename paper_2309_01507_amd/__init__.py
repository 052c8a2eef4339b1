"""MI355X-native 4-bit AdamW step (arXiv 2309.01507): thin ctypes binding over lpmm4.so.

The library is loaded on first use; nothing here computes anything on the CPU.
"""
from .binding import (  # noqa: F401
    LpmmError, State4, lib, lib_path, build_library, GRAD_F32, GRAD_BF16,
    lpmm_table, lpmm_host_nearest_codes, lpmm_adamw4_workspace_bytes, lpmm_adamw4_init,
    lpmm_adamw4_state_sizes, lpmm_adamw4_state_zero, lpmm_adamw4_step, lpmm_adamw4_step_bf16g,
    lpmm_adamw4_step_noalloc, lpmm_adamw4_step_ws, lpmm_ablation_table, lpmm_quant_ablation, lpmm_dequant_ablation,
    ablation_scale_sizes, NORM_B128, NORM_B2048, NORM_RANK1, MAP_DE, MAP_DE0, MAP_LINEAR, ROUND_NEAREST, ROUND_STOCHASTIC,
    lpmm_adamw32_step, lpmm_dequant_state, lpmm_quant_state, ensure_init, new_state,
    lpmm_profile_begin, lpmm_profile_end, TensorDesc, make_desc, new_plan, KIND_4BIT, KIND_FP32,
    lpmm_adamw4_plan_bytes, lpmm_adamw4_plan_build, lpmm_adamw4_step_multi, lpmm_adamw4_plan_release,
    StateB128, new_state_b128, KIND_4BIT_B128, lpmm_adamw4_b128_state_sizes, lpmm_adamw4_b128_state_zero,
    lpmm_adamw4_b128_step, lpmm_adamw4_b128_step_bf16g,
    StateFactor, new_state_factor, lpmm_adamw4_factor_state_sizes, lpmm_adamw4_factor_state_zero,
    lpmm_adamw4_factor_step, lpmm_adamw4_factor_step_bf16g, KIND_4BIT_FACTOR,
    StateND, new_state_nd, lpmm_adamw4_nd_state_sizes, lpmm_adamw4_nd_state_zero, lpmm_adamw4_nd_step,
    lpmm_adamw4_nd_step_bf16g,
    StateSgdm, new_state_sgdm, lpmm_sgdm4_state_sizes, lpmm_sgdm4_state_zero, lpmm_sgdm4_step, lpmm_sgdm4_step_bf16g,
    lpmm_sgdm32_step, lpmm_sgdm4_step_multi, make_desc_sgdm, lpmm_adamw4_step_multi_capturable,
    lpmm_sgdm4_step_multi_capturable, KIND_SGDM_4BIT, KIND_SGDM_FP32, FLAG_NO_DECAY, FLAG_DETERMINISTIC, KIND_4BIT_ND,
)
from .optim import AdamW4bit, SGDM4bit  # noqa: F401,E402
