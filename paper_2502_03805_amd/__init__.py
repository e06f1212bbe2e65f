"""MI355X-native per-layer KV-cache selection pass (score -> select -> compact).

The compute lives in libcriticalkv.so (hand-written gfx950 HIP kernels behind the C ABI of
include/criticalkv.h); this package is its ctypes binding.
"""
from .binding import (CKV_BF16, CKV_F32, CKV_MEAN, CKV_SUM, CKV_NORM_L1, CKV_NORM_L2, CKV_WO_OUT_IN, CKV_NO_MFMA, CKV_WO_IS_GRAM, CKV_CAUSAL_TAIL, CKV_PROTECT_WINDOW, CKV_ATTN_ONLY, criticalkv_prepare_gram, criticalkv_allocate, criticalkv_diagnostics, DIAG_FIELDS, gram_bytes,  # noqa: F401
                      CKV_OK, CKV_E_INVALID_ARG, CKV_E_UNSUPPORTED, CKV_E_WORKSPACE, CKV_E_HIP, CKV_E_STATIC_LIMIT,
                      CKV_STATIC_SCRATCH_BYTES, EXPORTS, criticalkv_select_noalloc, criticalkv_prepare_wo, prepared_wo_bytes,
                      criticalkv_probe_mfma_bf16, criticalkv_probe_hbm_read,
                      CriticalKVError, LayerDesc, hip_runtime, criticalkv_compact, criticalkv_score, criticalkv_score_profiled, criticalkv_select, load, STAGES,
                      make_desc, strerror, workspace_bytes)
