"""HCAttention decode hot path for MI355X: HIP kernels behind a C ABI (libhca.so) and a thin
ctypes binding with the same names."""
from .binding import (HcaError, hca_attend_gathered, hca_evict, hca_gather_values, hca_export_kcache, hca_kcache_bytes, hca_quantize_keys,  # noqa: F401
                      hca_score_qkeys, hca_shape, hca_sparse_attend, hca_topk, hca_version,
                      hca_workspace_bytes, lib, make_shape, hca_layer, hca_pipeline_desc, hca_pipeline_create,
                      hca_pipeline_destroy, hca_pipeline_step, hca_pipeline_scan_ms, hca_tune, hca_scan_stamp_pairs,
                      hca_wall_clock_khz)
