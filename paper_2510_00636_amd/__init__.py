"""MI355X-native Expected-Attention KV-cache compression: thin Python binding over libea.so.

Every step of the path runs in the HIP kernels of the shared library; this package only
marshals arguments (pointers, sizes, the stream).  There is no CPU or PyTorch fallback: if the
library is missing, importing `binding` functions raises."""
from .binding import (EaError, EaParams, make_params, workspace_bytes, query_stats, query_stats_hidden, score, wo_gram, value_norms_wo, score_wo, select, select_static,  # noqa: F401
                      compact, compact_unordered, select_adaptive, compact_ragged, compress_layer_adaptive, score_baseline, SCORER_KNORM, SCORER_STREAMING, SCORER_KEYDIFF, compress_layer, compress_layer_unordered, compress_layer_timed, debug_status, EaPaged, make_paged, score_paged, compact_paged, compress_layer_paged, score_fp8, compress_layer_fp8, EA_FP8_E4M3, STAGE_NAMES,
                      STATUS_BAD_SCORE, STATUS_COMPACT_WAIT, STATUS_BAD_INDEX, n_keep, status_string, lib_path, load_library,
                      EA_F32, EA_BF16)
