"""MI355X-native FlashMask attention (arXiv 2410.01359): thin Python binding
over the C-ABI HIP library.  Every step of the path runs in the HIP kernels;
this package only marshals arguments and owns device memory through torch."""
from .binding import (  # noqa: F401
    FM_PASS_BWD, FM_PASS_BWD_DKDV, FM_PASS_BWD_DQ, FM_PASS_FWD,
    FlashMaskError, Strides, flashmask_bwd, flashmask_bwd_ex, flashmask_classify, flashmask_fwd, flashmask_fwd_ex, flashmask_fwd_noalloc, flashmask_mfma_ceiling, flashmask_atomic_ceiling,
    flashmask_preprocess, flashmask_tile_shape, flashmask_unit_queues, flashmask_workspace_bytes,
    library_path, load_library,
)
