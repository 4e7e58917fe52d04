"""MI355X-native cross-layer attention-similarity estimator and layer-pair selector
(the data-parallel core of Krul, arxiv 2507.08045).  The work is done by
libkrul.so (HIP, gfx950); see include/krul.h for the C ABI and binding.py for the
thin Python layer over it."""
from .binding import (KRUL_BF16, KRUL_EDTYPE, KRUL_EINVAL, KRUL_ELAUNCH, KRUL_ESCRATCH, KRUL_STATIC_SCRATCH_BYTES, KRUL_EUNSUPPORTED, KRUL_EWORKSPACE,
                      KRUL_F16, KRUL_F32, KRUL_FLAG_CAUSAL, KRUL_FLAG_GENERIC_KERNEL, KRUL_FLAG_SINGLE_SPLIT,
                      KRUL_OK, KrulError, KrulKLayout, KrulKPages, KrulKeys, KrulShape, PagedKeys,
                      StridedKeys, all_pairs_similarity, all_pairs_similarity_in_place,
                      all_pairs_workspace_bytes, calibration_block, calibration_copy, lib, plan,
                      make_shape, n_select_from_ratio, pair_scores_from_sums, pair_similarity,
                      pair_similarity_accumulate, pair_similarity_accumulate_in_place, pair_similarity_ir,
                      pair_similarity_ir_in_place, pair_similarity_paged, pair_similarity_select, pair_similarity_static,
                      pair_similarity_strided, select_pairs, select_pairs_all, strerror, workspace_bytes,
                      workspace_bytes_ir)  # noqa: F401
