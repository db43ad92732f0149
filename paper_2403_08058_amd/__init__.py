"""MI355X-native clustered-head decode attention (CHAI): Python face of the C-ABI library libchai.so."""
from .binding import (CHAI_BF16, CHAI_F32, CHAI_OK, EXPORTS, LIB_PATH, ChaiError, alloc_workspace, chai_append_kv,
                      chai_assign_clusters, chai_compact_kcache, chai_decode_attention, chai_decode_scores, chai_decode_scores_timed, chai_decode_values, chai_decode_values_timed, chai_decode_workspace_bytes,
                      chai_dense_decode_attention, chai_score_features, chai_status_string, chai_version, lib)

__all__ = ["CHAI_BF16", "CHAI_F32", "CHAI_OK", "EXPORTS", "LIB_PATH", "ChaiError", "alloc_workspace",
           "chai_append_kv", "chai_assign_clusters", "chai_compact_kcache", "chai_decode_attention",
           "chai_decode_scores", "chai_decode_scores_timed", "chai_decode_values", "chai_decode_values_timed", "chai_decode_workspace_bytes", "chai_dense_decode_attention", "chai_score_features",
           "chai_status_string", "chai_version", "lib"]
