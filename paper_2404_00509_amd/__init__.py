"""MI355X-native MAE input pipeline and normalised-pixel loss (DailyMAE, arXiv 2404.00509).

The work is done by ``libmae_hip.so`` (hand-written HIP for gfx950 behind a C ABI, declared in
``include/mae_hip.h``); this package is the thin binding with the same entry-point names.
Importing the package does not load the library; the first call does, and raises if it is absent.
"""
from .binding import (  # noqa: F401
    EXPORTS,
    IMAGENET_MEAN,
    IMAGENET_STD,
    LIB_PATH,
    MAE_AUG_SIMPLE,
    MAE_AUG_THREE,
    MAE_AUG_THREE_PLUS,
    MAE_BF16,
    MAE_F32,
    MAE_INPUT_DECODED,
    MAE_INPUT_JPEG,
    MaeEmbedDesc,
    MaeError,
    MaeLossDesc,
    MaePrepDesc,
    PrepBuffers,
    ProgressiveBuffers,
    alloc_prep_buffers,
    load,
    mae_error_string,
    mae_finetune_stage,
    mae_pretrain_stage,
    mae_stage_of_epoch,
    mae_loss_from_images_workspace_bytes,
    mae_loss_workspace_bytes,
    mae_normpix_loss,
    mae_normpix_loss_from_images,
    mae_num_keep,
    mae_patch_embed,
    mae_prep_batch,
    mae_prep_status,
    mae_prep_workspace_bytes,
    mae_version,
    make_embed_desc,
    make_loss_desc,
    make_prep_desc,
)
