"""MI355X (gfx950) implementation of one Block Selective Reprogramming fine-tuning step
(arxiv 2405.10951).  All arithmetic runs in the HIP kernels of libbsr_hip.so behind the C ABI of
include/bsr.h; this package only marshals arguments.  There is no CPU fallback: importing works
anywhere, calling anything needs the built library and a gfx950 device."""
from .binding import (BSR_BF16, BSR_FP32, BSR_LOSS_CE, BSR_LOSS_MEAN_SQ, BsrError, Context,  # noqa: F401
                      bsr_attention_backward, bsr_attention_forward, bsr_gemm_tile_shapes, bsr_linear_dgrad, bsr_linear_forward, bsr_linear_wgrad, bsr_linear_wgrad_static,
                      bsr_ln_linear_fold, bsr_ln_linear_forward, bsr_saved_activation_bytes, bsr_token_schedule,
                      bsr_workspace_bytes, lib_path, load_library, make_config)
