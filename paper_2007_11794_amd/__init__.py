"""MI355X-native batched RNNLM scoring step (dedup -> hidden update -> fused output
projection + log-sum-exp -> query gather) behind a C ABI; this package is the thin Python
binding over librnnlm.so.  PyTorch is used only for device memory and streams."""
from .binding import (RNNLM_BF16, RNNLM_F32, FLAG_BAD_PREV_WORD, FLAG_BAD_QUERY_WORD, FLAG_BAD_ROW,
                      OPT_LSE_MODE, OPT_OUTPROJ_KERNEL, RnnlmError, RnnlmModel, lib, lib_path,
                      rnnlm_dedup, rnnlm_dedup_static, DEDUP_STATIC_MAX_N, rnnlm_dedup_workspace_bytes, rnnlm_load, rnnlm_step,
                      rnnlm_step_dedup, rnnlm_strerror, RnnlmCache, rnnlm_cache_create,
                      rnnlm_step_cached, rnnlm_pack_ids, RnnlmIndexTable, rnnlm_index_create,
                      rnnlm_index_intern, rnnlm_index_fetch, INDEX_NOT_STORED, INDEX_COLLISION,
                      rnnlm_huffman_build, rnnlm_hs_load, rnnlm_hs_step, rnnlm_hs_time_query,
                      rnnlm_probe_mfma_rate, rnnlm_time_empty_launch)

__all__ = ["RNNLM_BF16", "RNNLM_F32", "FLAG_BAD_PREV_WORD", "FLAG_BAD_QUERY_WORD", "FLAG_BAD_ROW",
           "OPT_LSE_MODE", "OPT_OUTPROJ_KERNEL", "RnnlmError", "RnnlmModel", "lib", "lib_path",
           "rnnlm_dedup", "rnnlm_dedup_static", "DEDUP_STATIC_MAX_N", "rnnlm_dedup_workspace_bytes", "rnnlm_load", "rnnlm_step",
           "rnnlm_step_dedup", "rnnlm_strerror", "RnnlmCache", "rnnlm_cache_create",
           "rnnlm_step_cached", "rnnlm_pack_ids", "RnnlmIndexTable", "rnnlm_index_create",
           "rnnlm_index_intern", "rnnlm_index_fetch", "INDEX_NOT_STORED", "INDEX_COLLISION",
           "rnnlm_huffman_build", "rnnlm_hs_load", "rnnlm_hs_step", "rnnlm_hs_time_query",
           "rnnlm_probe_mfma_rate", "rnnlm_time_empty_launch"]
