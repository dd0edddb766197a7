"""MI355X-native vocabulary layers of Vocabulary Parallelism (arXiv 2411.05288).

The product is libvp.so (HIP kernels behind a C ABI, see include/vp.h).  This package is
the thin Python binding over it: argument marshalling only, every step of the path runs
in the library's kernels.  PyTorch supplies device memory and streams.
"""
from .binding import (  # noqa: F401
    VP_BF16, VP_F32, VP_SAVE_LOGITS, VP_SKIP_DH, VP_DH_OVERWRITE, VPError, lib_path, load_library,
    vp_combine_stats, vp_dlogits_row_stride, vp_embed_bwd, vp_embed_fwd, vp_output_bwd, vp_output_dx_alg2, vp_output_fwd, vp_output_fwd_alg2, vp_output_fwd_noalloc,
    vp_output_fwd_noalloc_max_scratch,
    vp_profile_enable, vp_profile_force_generic_gemm, vp_profile_gemm_trace, vp_profile_mfma_loop, vp_profile_mfma_variant, vp_profile_mfma_variant_count, vp_profile_read, vp_version, vp_workspace_bytes,
)
from . import driver  # noqa: F401
from .driver import (  # noqa: F401
    EmbeddingPlan, OutputLayerPlan, OutputLayerResult, embedding_backward, embedding_forward, output_layer_step,
)
