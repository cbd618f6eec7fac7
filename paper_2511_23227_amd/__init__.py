"""pcpp: PointCNN++ convolution on native points as MVMR, hand-written HIP for MI355X (gfx950).

The package is a thin ctypes binding over libpcpp.so (see include/pcpp.h).  Every step of the
path -- hashed-grid radius search, reordering by (k, o), MVMR forward and both gradients -- runs
in the library's kernels; PyTorch only provides device memory and the stream.
"""
from . import binding
from .binding import (BUILD_TEST_SHORT_LISTS, BUILD_TEST_WIDE_KEYS, BUILD_VOXEL, PLAN_BWD_INPUT, PLAN_FWD, PLAN_SPATIAL, PcppError,
                      Triplets, library, pcpp_build_triplets, pcpp_count_triplets, pcpp_mvmr_bwd_input,
                      pcpp_mvmr_bwd_weight, pcpp_mvmr_fwd, pcpp_mvmr_fwd_static, pcpp_tune_plan_order, pcpp_voxel_subsample)

__all__ = ["BUILD_TEST_SHORT_LISTS", "BUILD_TEST_WIDE_KEYS", "BUILD_VOXEL", "pcpp_voxel_subsample", "PLAN_BWD_INPUT", "PLAN_FWD", "PLAN_SPATIAL", "PcppError",
           "Triplets", "binding", "library", "pcpp_build_triplets", "pcpp_count_triplets", "pcpp_mvmr_bwd_input",
           "pcpp_mvmr_bwd_weight", "pcpp_mvmr_fwd", "pcpp_mvmr_fwd_static", "pcpp_tune_plan_order"]
