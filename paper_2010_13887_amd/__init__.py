"""MI355X-native beam-search Transformer decoding (LightSeq's hot path, arxiv 2010.13887).

The product is ``liblsq.so`` (hand-written HIP for gfx950 behind a C ABI, see include/lsq.h).
This package is a thin ctypes binding with the same call names; PyTorch is used only to own
the device workspace and the stream.  There is no CPU fallback: without the built library every
call raises.
"""
from .binding import (LsqError, Engine, load_library, library_path, lsq_workspace_bytes,  # noqa: F401
                      lsq_set_workspace, lsq_init, lsq_encode, lsq_decode_step, lsq_decode_steps,
                      lsq_get_beams, lsq_free, lsq_last_error, lsq_step_index, lsq_set_graphs, lsq_set_cache_refresh, lsq_set_diversity, lsq_set_layernorm_fusion, lsq_set_attention_blocks, lsq_set_topk_statistics, lsq_set_canaries, lsq_debug_check_canaries, k_layernorm_gemm, k_layernorm_cross_attention, k_cross_attention_q, k_self_attention_block, k_cross_attention_block, k_gemm_logits, k_gemm_logits_supported, k_row_topk_groups,
                      REFRESH_MOVE, REFRESH_TABLE, lsq_debug_read, lsq_profile_enable, lsq_profile_read,
                      k_gemm, k_pack_weights, k_gemm_add_layernorm, k_gemm_add_layernorm_static, k_gemm_add_layernorm_static_limit, k_self_attention, k_self_attention_table, k_encoder_attention, k_cross_attention, k_row_topk,
                      k_beam_refine, k_cache_reorder, DBG)
