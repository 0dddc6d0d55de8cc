"""MI355X-native hot path of QwT-v2: W8A8 quantized linear layer with the folded
channel-wise affine compensation in its GEMM epilogue, and the calibration
statistics / closed-form fit / fold that produce its parameters.

``binding`` exposes the C-ABI entry points of libcwac_hip.so one to one;
``synth`` draws the seeded synthetic workloads."""
from . import synth  # noqa: F401
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    CWAC_EPI_FP_BIAS, CWAC_EPI_INT_OFFSET, CWAC_OUT_FP32, CWAC_OUT_INT8, CWAC_OUT_INT32,
    CwacError, cwac_apply_unfolded, cwac_calibrate_stats, cwac_calibrate_stats_workspace,
    cwac_colsum, cwac_epilogue_int32, cwac_fold, cwac_qparams, cwac_qparams_from_range,
    cwac_quantize_act, cwac_quantize_rows_sym, cwac_range_f32, cwac_range_workspace, cwac_solve,
    cwac_stats_bytes, cwac_stats_reset, make_qparams, qlinear_cwac_forward,
    cwac_calibrate_stats_first, cwac_tuning, make_tuning, cwac_calibrate_stats_static, cwac_static_scratch_bytes,
    cwac_calibrate_fused_workspace, qlinear_cwac_calibrate_fused, cwac_mfma_probe, cwac_mfma_probe_f16, cwac_hbm_read_probe, cwac_kloop_probe,
    cwac_fold_fixed_point, qlinear_cwac_forward_fixed_point,
    cwac_quantize_act_bits, cwac_quantize_rows_sym_bits,
    CWAC_OUT_FP16, CWAC_W4_GROUP, cwac_w4_quantize_groupwise, cwac_w4_packed_w_bytes, cwac_w4_pack,
    cwac_fold_weight_only, qlinear_w4a16_cwac_forward, qconv2d_cwac_forward,
    vit_residual_ln_quant, vit_gelu_table, vit_table_lookup, vit_attention_int8,
    qlinear_cwac_forward_table, vit_block_workspace, vit_block_w8a8_forward, vit_encoder_w8a8_forward, vit_block_params, vit_block_layer, make_block_params,
)
