"""MI355X-native intermediate-layer token recall (ILRe, Section 3.2): Python binding of libilre."""
from .binding import (ILRE_BF16, ILRE_EHIP, ILRE_EINVAL, ILRE_ENOMEM, ILRE_EUNSUPPORTED, ILRE_F32, ILRE_FLAG_EXACT_ROW_MAX,
                      ILRE_MAX_AVG_KERNEL, ILRE_MAX_BUDGET, ILRE_MAX_MAX_KERNEL, ILRE_MAX_POOL_KERNEL, ILRE_ROPE_HALF, ILRE_ROPE_INTERLEAVED, ILRE_MAX_POOL_KERNELS, ILRE_OK, ILRE_SCORE_MAX,
                      ILRE_SCORE_SUM, EXPORTS, IlreError, IlreOpts, alloc_workspace, ilre_col_scores, ilre_gather_ids,
                      alloc_workspace_max_avg, ilre_last_error, ilre_recall, ilre_recall_max_avg, ilre_rerope_keys, ilre_probe_describe, ilre_probe_mfma_ceiling, ILRE_PROBE_OPERAND_BYTES, ILRE_PROBE_OUT_BYTES, ilre_row_stats, ilre_row_stats_static, ilre_select, ILRE_STATIC_SCRATCH_BYTES,
                      ilre_select_max_avg, ilre_workspace_bytes, ilre_workspace_bytes_max_avg, load, to_device)

__all__ = [n for n in dir() if n.startswith(("ilre_", "ILRE_", "Ilre"))] + ["alloc_workspace", "alloc_workspace_max_avg", "load", "to_device", "EXPORTS"]
