"""MI355X-native KurTail rotation-learning step: thin Python binding.

Argument marshalling only.  Every step of the path runs in the HIP kernels of
``libkurtail.so`` (see ``include/kt.h`` for the C ABI); PyTorch is used for device
memory and the current stream.  There is no CPU or eager fallback: if the library
has not been built, importing the binding functions raises.
"""
from .binding import (  # noqa: F401
    KT_F32,
    KT_BF16,
    KT_OP_LOSS_GRAD,
    KT_OP_CAYLEY,
    KT_OP_FAKEQUANT,
    KT_OP_POOLED_LOSS_GRAD,
    KT_OP_QUANT_METRICS,
    KT_OP_FUSE_ROTATION,
    KT_OP_SENSITIVITY,
    KT_OP_LOSS_GRAD_RECOMPUTE,
    KT_OP_POOLED_LOSS_GRAD_RECOMPUTE,
    KtError,
    lib,
    lib_path,
    kt_version,
    kt_last_error,
    kt_workspace_bytes,
    kt_kurtosis_loss_grad,
    kt_pooled_kurtosis_loss_grad,
    kt_cayley_step,
    kt_cayley_step_static,
    kt_cayley_adam_step,
    kt_rotate_fakequant_int4,
    kt_rotate_quant_metrics,
    kt_hadamard_rows,
    kt_fuse_rotation,
    kt_quant_sensitivity,
    Workspace,
    kt_profile_enable,
    kt_profile_read,
    kt_profile_reset,
)
