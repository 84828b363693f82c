"""MI355X (gfx950) implementation of one MoHGE layer (forward, auxiliary losses, backward)
behind a C ABI.

`binding` marshals torch tensors into the calls of `include/mohge.h`; every step
of the layer runs in the HIP kernels of `csrc/`.  There is no CPU or PyTorch fallback:
if `libmohge.so` has not been built, loading fails.
"""
from .binding import (  # noqa: F401
    MohgeError, Config, lib, lib_path, mohge_route, mohge_permute, mohge_permute_static, mohge_expert_ffn, mohge_expert_ffn_up, mohge_expert_ffn_down,
    mohge_combine, mohge_aux_loss, mohge_workspace_size, mohge_last_error, pack_w13,
    MoHGELayer, CALL_PERMUTE, CALL_EXPERT_FFN, CALL_AUX_LOSS, SELECT_GLOBAL, SELECT_PER_GROUP,
    F32, BF16, CALL_FFN_SAVED, CALL_EXPERT_FFN_BWD, CALL_ROUTE_BWD, CALL_ROUTE, mohge_expert_ffn_train,
    mohge_combine_bwd, mohge_expert_ffn_bwd, mohge_route_bwd,
    mohge_shared_routing, mohge_combine_add, SharedExperts, mohge_expert_ffn_w8, mohge_fp8_decode,
    mohge_fused_status, mohge_expert_ffn_w4, mohge_mxfp4_decode, mohge_decode_layer,
    mohge_decode_layer_ctl_bytes, CALL_DECODE_LAYER,
)
from .weights import quantize_rows_e4m3, quantize_mxfp4  # noqa: F401
