"""MI355X (gfx950) implementation of one T5.1.1-style Transformer block (encoder layer, decoder-only
layer, or decoder layer with cross-attention): forward, backward, relative-position buckets and the
Adafactor update, behind the C ABI of include/t5mi.h.

Python here only marshals arguments: every arithmetic step runs in the HIP kernels of libt5mi.so.
"""
from .binding import (  # noqa: F401
    T5Error,
    CROSS_WEIGHT_NAMES,
    WEIGHT_NAMES,
    adafactor_step,
    adafactor_step_multi,
    adafactor_step_static,
    adafactor_multi_workspace_bytes,
    adafactor_workspace_bytes,
    lib,
    lib_path,
    t5_block_bwd,
    t5_block_fwd,
    t5_block_kernel_path,
    PATH_MFMA_GEMM,
    PATH_MFMA_ATTN_FWD,
    PATH_MFMA_ATTN_BWD,
    PATH_MFMA_CROSS_ATTN,
    t5_block_stash_bytes,
    t5_block_workspace_bytes,
    t5_decoder_block_bwd,
    t5_decoder_block_fwd,
    t5_decoder_block_stash_bytes,
    t5_decoder_block_workspace_bytes,
    t5_dropout_keep,
    t5_wgrad_overlap_enable,
    t5_encdec_loss_and_grad,
    t5_encdec_workspace_bytes,
    t5_gemm_bf16,
    t5_stack_loss_and_grad,
    t5_stack_workspace_bytes,
    t5_mfma_peak_probe,
    t5_relpos_bucket,
    t5_step_timing_enable,
    t5_step_timing_read,
    t5_status_string,
)
