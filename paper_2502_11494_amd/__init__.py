"""DART token reduction (arXiv 2502.11494, Section 3.3) for MI355X: hand-written
HIP kernels behind the C ABI of include/dart.h, with a ctypes binding."""
from .binding import (DART_BF16, DART_ERR_ALIGN, DART_ERR_BUDGET, DART_ERR_DEVICE,  # noqa: F401
                      DART_ERR_DTYPE, DART_ERR_HIP, DART_ERR_NULL, DART_ERR_SHAPE,
                      DART_ERR_STATIC_LIMIT,
                      DART_ERR_WORKSPACE, DART_F32, DART_OK, DART_PIVOT_MAX_L1,
                      DART_PIVOT_GIVEN, DART_PIVOT_MIN_L1, DART_PIVOT_RANDOM, DART_SCORE_MAX, DART_SCORE_MIN,
                      DART_SCORE_PER_PIVOT, DartDesc, DartError, DartRowTensor, alloc_workspace,
                      dart_compact_sequences,
                      dart_device_status, dart_duplication_scores, dart_gather_compact,
                      dart_device_status_static, dart_probe_mfma_dot32, dart_reduce,
                      dart_reduce_profiled, dart_reduce_static, dart_reduce_with_norms,
                      dart_score_tile_shape,
                      dart_score_tile_shape_first_read,
                      dart_select_pivots,
                      dart_static_scratch_bytes, dart_topk_keep,
                      dart_workspace_bytes, make_desc, score_tolerance, strerror)
