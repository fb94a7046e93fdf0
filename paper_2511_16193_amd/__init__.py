"""MI355X-native batched speculative-verification step (C-ABI library + thin binding).

The product is paper_2511_16193_amd/libspecverify.so (HIP, gfx950); this package only
marshals arguments.  There is no CPU fallback: using the binding without the built
library raises.
"""
from .binding import (Verifier, SvError, lib, load_library, op_gemm_bf16, op_gemm_bf16_ws, op_gemm_plan, op_pack_rows, op_pack_weight, pack_weights, op_sample, EXPORTS, LIB_PATH,  # noqa: F401
                      SV_FP32, SV_BF16, SV_GREEDY, SV_STOCHASTIC, SV_MATCH, SV_INVERSE_CDF, SV_EXP_RACE, SV_OPT_GEMM_VARIANT, SV_OPT_ATTN_GENERIC, SV_OPT_ATTN_MIN_ROW_TILES, SV_OPT_ATTN_CHUNK_KEYS, SV_OPT_ATTN_MAX_ROW_TILES, SV_OPT_GRAPH, SV_OPT_GEMM_TILE, SV_PROF_GEMM, SV_PROF_ATTENTION,
                      SV_PROF_SAMPLER, SV_PROF_ROLLBACK, SV_PROF_MOE, op_moe_ffn,
                      op_sample_static, probe_peaks, probe_copy, probe_mfma_valu, plan_accept_prob, plan_tau, plan_decoupled, plan_best_window, fit_affine)
