// Fitted coefficients of the selector's latency estimates (microseconds per term), in the order of the term
// enumerations of tdc_select.cpp.  Written by
//     python -m paper_2211_03715_amd.autotune --fit <sweeps.json ...> --write-coef
// from exhaustive sweeps timed on MI355X (`--out` of the same module); do not edit by hand.
#ifndef TDC_SELECT_COEF_H
#define TDC_SELECT_COEF_H

// fused, latency regime: launch s1_unit s1_kg s1_mfma s1r_unit s1r_kg s1r_mfma s2_kg_lds s2_kg_glb s2_mfma s3_unit s3_kg_lds s3_kg_glb s3_mfma w_kb x_mb_nchw x_mb_nhwc x_mb_runs y_mb_nchw y_mb_nhwc x_rows y_rows
static const double kFusedLatencyCoef[22] = {3.0025, 0.1184, 0, 0.0828, 0, 0, 0, 0.1051, 0.1331, 0.0037, 0.1798, 0.0151, 0, 0.1193, 0.0166, 42.3792, 28.4607, 0, 7.0969, 0, 0.9402, 0};
// fused, throughput regime: same terms
static const double kFusedThroughputCoef[22] = {3.8605, 0, 0.0988, 0.0347, 0.6828, 0.1891, 0.0176, 0.0560, 0.0826, 0.0210, 0.1531, 0.0330, 0.0167, 0.1457, 0.0207, 19.2123, 11.7344, 6.1081, 48.2178, 30.6810, 0.2834, 0.4272};
// chain: launch s1_unit s1_kg s1_mfma s1r_unit s1r_kg s1r_mfma kg2_lds kg2_glb blk2 nb3_lds blk3 w_kb x_mb_nchw x_mb_nhwc x_mb_runs y_mb x_rows y_rows novec
static const double kChainCoef[20] = {3.6918, 0.5859, 0.0211, 0.0906, 0.2783, 0.3798, 0.0096, 0.0298, 0.2335, 0.0141, 0.2690, 0.0402, 0.0235, 6.4658, 0, 15.9944, 32.4026, 0.2683, 2.9056, 0.1707};
// fused-merged: launch s1_unit s1_kg s1_mfma frag reduce x_mb_nchw x_mb_nhwc wgs
static const double kFmCoef[9] = {2.5879, 0.2174, 0.0197, 0.0407, 0.0803, 0.4477, 38.3935, 16.4747, 0.5418};
// one GEMM launch (split, merged, dense): launch wave kg mfma conv_b reduce act_1x1 act_conv
static const double kStageCoef[8] = {2.15, 0.05, 0.0649, 0.0785, 0.0255, 0.3158, 0.0653, 0.0246};
// the dense K x K layer (one GEMM launch that writes y): the eight terms above, then y_nchw y_nhwc
static const double kDenseCoef[10] = {2.4298, 0.0481, 0.0128, 0.0674, 0.0376, 0.3898, 0, 0.0158, 0.1439, 0.0498};

#endif
