"""MI355X (gfx950) forward convolution and SGEMM behind the C ABI of include/polydl.h.

The Python layer only marshals arguments (device pointers, sizes, the current HIP stream) into
libpolydl.so; every arithmetic step runs in the HIP kernels.  There is no CPU fallback: if the
library has not been built, importing this package raises.
"""
from .binding import (lib, PolydlError, TileCfg, ACT, conv2d_fwd, conv2d_fwd_noalloc, filter_tap_copy, sgemm, set_tile_override,
                      get_last_tile, variants, status_string, LIB_PATH, nchw_to_nchwc,
                      nchwc_to_nchw, kcrs_to_kcrsck, bias_add, activation, ModelReport,
                      reuse_bucket, reuse_cost, model_get_levels, model_set_levels, model_conv2d, model_sgemm, pick_conv2d, pick_sgemm,
                      conv_candidates, nchw_to_nchwc_bf16, kcrs_to_kcrsck_bf16, conv2d_fwd_bf16_blocked,
                      conv2d_fwd_bf16, bnorm_fwd, model_conv2d_bf16, pick_conv2d_bf16,
                      conv_candidates_bf16, sgemm_candidates, ranker_num_params, ranker_set_params,
                      ranker_load, ranker_stats_conv2d, ranker_play, ranker_tournament, pick_conv2d_learned,
                      RANKER_STATS, RANKER_PARAMS_PATH, reuse_analyse)

__all__ = ["lib", "PolydlError", "TileCfg", "ACT", "conv2d_fwd", "conv2d_fwd_noalloc", "filter_tap_copy", "sgemm", "set_tile_override",
           "get_last_tile", "variants", "status_string", "LIB_PATH", "nchw_to_nchwc", "nchwc_to_nchw",
           "kcrs_to_kcrsck", "bias_add", "activation", "ModelReport", "reuse_bucket", "reuse_cost",
           "model_get_levels", "model_set_levels", "model_conv2d", "model_sgemm", "pick_conv2d", "pick_sgemm", "conv_candidates",
           "nchw_to_nchwc_bf16", "kcrs_to_kcrsck_bf16", "conv2d_fwd_bf16_blocked", "conv2d_fwd_bf16", "bnorm_fwd",
           "model_conv2d_bf16", "pick_conv2d_bf16", "conv_candidates_bf16", "sgemm_candidates",
           "ranker_num_params", "ranker_set_params", "ranker_load", "ranker_stats_conv2d", "ranker_play",
           "ranker_tournament", "pick_conv2d_learned", "RANKER_STATS", "RANKER_PARAMS_PATH", "reuse_analyse"]
