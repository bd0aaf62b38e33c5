"""MI355X-native hot path of SURGEON's adaptation step (layer-wise dynamic activation pruning).

Everything is computed by hand-written HIP kernels in ``libsurgeon.so`` behind a C ABI (``include/surgeon.h``);
this package only marshals arguments.  PyTorch is used for device memory and streams.
"""
from .binding import (  # noqa: F401
    BF16,
    F32,
    LayerDesc,
    PackedActivation,
    SurgeonError,
    conv2d_desc,
    dw_from_packed,
    grad_importance,
    library_path,
    linear_desc,
    load_library,
    prune_pack,
    surgeon_dw_from_packed,
    surgeon_dw_kernel_class,
    surgeon_dw_ws_bytes,
    surgeon_grad_importance,
    surgeon_grad_importance_batched,
    surgeon_grad_importance_batched_ws_bytes,
    surgeon_grad_importance_static,
    surgeon_grad_importance_ws_bytes,
    surgeon_keep_count,
    surgeon_last_error,
    surgeon_layer_ratios,
    surgeon_packed_sizes,
    surgeon_prune_pack,
    surgeon_profile_begin,
    surgeon_profile_end,
    surgeon_version,
)
