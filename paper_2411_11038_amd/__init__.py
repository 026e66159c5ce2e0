"""Python binding of libefqat.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (torch is used for device
memory and streams, nothing else), passes their pointers through the C ABI declared in
include/efqat.h and returns the library's outputs.  There is no CPU fallback: without the
built library (or without a GPU for the compute calls) these functions raise.
"""
from .binding import (  # noqa: F401
    EfqatError, lib, lib_path, k_from_ratio, fakequant_fwd, channel_select, channel_select_static, weight_quant_select, network_select,
    layer_select, bias_grad, linear_bwd, linear_bwd_weight_operand, conv_bwd, linear_fwd, F32, BF16, ACT_PER_TENSOR_ASYM,
    W_PER_ROW_SYM, DY_TOKEN_MAJOR, DY_CHANNEL_MAJOR, EXPORTS, OptStep, profile_enable, profile_read, DX_KERNEL_AUTO,
    DX_KERNEL_BF16, DX_KERNEL_INT8, DX_KERNEL_BF16_PINNED, PROF_DX, PROF_DW, PROF_FWD, PROF_PREP, PROF_FINISH,
    PROF_QUANT_ACT, PROF_QUANT_W, PROF_IMPORTANCE, PROF_TOPK, PROF_BIAS, PROF_CLASSES,
)
