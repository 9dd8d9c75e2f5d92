"""MI355X-native forward sparse convolution layer with attention (arXiv 1801.10585).

Thin Python binding over the C-ABI library libscnn.so (hand-written HIP for
gfx950).  PyTorch is used only for device memory and streams; every step of the
layer runs in the library's kernels.  There is no CPU fallback: importing works
anywhere, calling an operator without the built library or without a GPU raises.
"""
from .binding import (  # noqa: F401
    ABS,
    SIGNED,
    FLAG_BAD_COORD,
    FLAG_CAND_OVERFLOW,
    FLAG_OUT_OVERFLOW,
    FLAG_UNSORTED,
    ScnnError,
    ChainedLayer,
    attention_topk,
    calibration_copy,
    density_regulariser,
    prune_weights,
    k_from_rho,
    library_path,
    profile_collect,
    profile_enable,
    load_library,
    set_conv_path,
    last_conv_kernel,
    sparse_conv_bwd,
    sparse_conv_bwd_workspace,
    sparse_conv_fwd,
    sparse_conv_fwd_max_rows,
    sparse_conv_fwd_workspace,
    sparse_maxpool,
    sparse_relu,
    sparse_relu_static,
    sparse_relu_static_max_rows,
    sparse_to_dense,
    validate_rows,
    EXPORTED_SYMBOLS,
)
from .metrics import count_mac_nz, count_bwd_visits, algorithmic_bytes  # noqa: F401
