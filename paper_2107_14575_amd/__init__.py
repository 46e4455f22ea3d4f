"""MI355X-native stochastic gradient quantizer: the data-parallel hot path of DQ-SGD
(arXiv 2107.14575).  Every step of the path runs in hand-written HIP kernels behind the C ABI
declared in ``include/dq.h``; this package only marshals arguments (``binding``) and holds the
seeded synthetic workload generators (``workloads``)."""
from .binding import (  # noqa: F401
    DQError,
    alpha_est,
    comm_cost_bits,
    unpack_dequant_reduce_update,
    Plan,
    Widths,
    comm_cost_bits_per_tensor,
    packed_bytes_v,
    quantize_pack_v,
    select_bits_per_tensor,
    select_bits_per_worker,
    unpack_dequant_reduce_update_v,
    unpack_dequant_reduce_v,
    library_path,
    load_library,
    norm,
    norm_linf,
    norm_static_scratch,
    norm_static_scratch_max_bytes,
    bracketed_workspace_bytes,
    norm_bracket,
    norm_quantize_pack,
    norm_quantize_pack_bracketed,
    norm_quantize_pack_bracketed_v,
    norm_quantize_pack_v,
    quantize_pack,
    select_bits,
    select_bits_device,
    sign_majority,
    sign_pack,
    sign_reduce,
    select_bits_linf,
    unpack_dequant_reduce,
)

__all__ = ["DQError", "Plan", "Widths", "comm_cost_bits_per_tensor", "packed_bytes_v", "quantize_pack_v",
           "select_bits_per_tensor", "select_bits_per_worker", "unpack_dequant_reduce_update_v", "unpack_dequant_reduce_v", "alpha_est", "comm_cost_bits", "library_path", "load_library", "norm", "norm_linf", "norm_static_scratch", "norm_static_scratch_max_bytes", "norm_quantize_pack", "norm_quantize_pack_v", "norm_quantize_pack_bracketed", "norm_quantize_pack_bracketed_v", "bracketed_workspace_bytes", "norm_bracket",
           "quantize_pack", "select_bits", "select_bits_device", "select_bits_linf", "sign_majority", "sign_pack", "sign_reduce", "unpack_dequant_reduce",
           "unpack_dequant_reduce_update"]
