"""MI355X-native embedding-table hot path of DQRM (arXiv 2410.20046).

The product is the C-ABI library ``libdqrm.so`` (``include/dqrm.h``), built from
the HIP sources under ``csrc/``.  This package is its thin ctypes binding.
"""
from .binding import (  # noqa: F401
    DqrmError, Tables, StepBuffers, DenseModel, lib, EXPORTS,
    OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE_TOO_SMALL, ERR_INDEX_OUT_OF_RANGE, ERR_HIP, ERR_CAPACITY,
    ERR_BAD_OFFSETS, ERR_SCRATCH_LIMIT, NOALLOC_SCRATCH_BYTES, FWD_MASTER, FWD_PACKED, SEG_CHUNK, MAX_TABLE_LOOKUPS, MAX_TABLES, MAX_DIM, MAX_DEDUPE_BATCHES,
    dqrm_version, dqrm_find_scale, dqrm_pack_int4, dqrm_embbag_fwd, dqrm_embbag_bwd_workspace_bytes,
    dqrm_embbag_bwd, dqrm_embbag_bwd_noalloc, dqrm_dedupe, dqrm_dedupe_multi, dqrm_segment_sum, dqrm_segment_sum_multi, dqrm_quant_update, dqrm_grad_quant_int8,
    dqrm_grad_quant_int8_multi, dqrm_sparse_update, dqrm_check_status,
    dqrm_sparse_merge_workspace_bytes, dqrm_sparse_merge, dqrm_sparse_update_sums, dqrm_sparse_block_t,
    dqrm_fwd_bwd_step, dqrm_dense_workspace_bytes, dqrm_dense_step, dqrm_dense_param_count, dqrm_dense_step_quant,
    DenseQuant,
)
from .build import build_library  # noqa: F401
