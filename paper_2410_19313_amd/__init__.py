"""MI355X-native FP8-state AdamW step of COAT (arxiv 2410.19313): HIP kernels behind a C ABI
(include/coat.h) and this thin binding; also the activation quantizers of Sec. 5.2."""
from .binding import (CoatError, HParams, FLAG_EXPAND, FLAG_E5M2, FLAG_M_E5M2, FLAG_V_E5M2, FLAG_M_PLAIN, FLAG_V_PLAIN, FLAG_BF16_SCALE, FLAG_BF16_K, FLAG_PRECISE_DQ,
                      step_flags, SUPPORTED_GROUP_SIZES, EXPORTS,
                      make_hparams, n_groups, strerror, lib,
                      coat_fp8_adamw_step, coat_fp8_adamw_step_bf16w, coat_quant_group, coat_dequant_group,
                      coat_act_quant_group, coat_act_quant_tensor, coat_act_quant_tensor_from_group_amax,
                      coat_act_quant_tensor_static, coat_bench_copy_control, ACT_GROUP_SIZES,
                      ACT_WORKSPACE_FLOATS, act_workspace,
                      TensorDesc, MultiPlan, coat_multi_plan_build, coat_fp8_adamw_step_multi, coat_shard_range,
                      StepConsts, coat_step_consts_compute, step_consts_tensor, coat_fp8_adamw_step_multi_consts)

__all__ = ["CoatError", "HParams", "FLAG_EXPAND", "FLAG_E5M2", "FLAG_M_E5M2", "FLAG_V_E5M2", "FLAG_M_PLAIN",
           "FLAG_V_PLAIN", "FLAG_BF16_SCALE", "FLAG_BF16_K", "FLAG_PRECISE_DQ", "step_flags", "SUPPORTED_GROUP_SIZES", "EXPORTS", "make_hparams",
           "n_groups", "strerror", "lib", "coat_fp8_adamw_step", "coat_fp8_adamw_step_bf16w", "coat_quant_group", "coat_dequant_group",
           "coat_act_quant_group", "coat_act_quant_tensor", "coat_act_quant_tensor_from_group_amax",
           "coat_act_quant_tensor_static", "coat_bench_copy_control", "ACT_GROUP_SIZES", "ACT_WORKSPACE_FLOATS", "act_workspace",
           "TensorDesc", "MultiPlan", "coat_multi_plan_build", "coat_fp8_adamw_step_multi", "coat_shard_range",
           "StepConsts", "coat_step_consts_compute", "step_consts_tensor", "coat_fp8_adamw_step_multi_consts"]
