"""ulsnn: fp32 SGEMM and the one-hidden-layer MLP gradient on AMD MI355X (gfx950).

A thin binding over the C ABI of libulsnn.so (include/ulsnn.h).  Every step of the path runs in the library's
HIP kernels; this package only marshals arguments.  PyTorch is used for device memory and streams.
"""
from .binding import (  # noqa: F401
    MlpGradResult,
    UlsnnError,
    lib_path,
    load,
    mlp_grad,
    mlp_grad_describe_plan,
    sgemm_describe_plan,
    dot,
    axpy,
    cg_direction,
    mlp_line_search,
    mlp_line_search_workspace_bytes,
    LineSearchResult,
    VEC_WORKSPACE_BYTES,
    sgemm_planned,
    TILE_SHAPES,
    mlp_grad_epoch,
    mlp_grad_flops,
    mlp_grad_mse,
    mlp_loss,
    mlp_loss_flops,
    mlp_mse,
    mlp_grad_timed,
    MLP_STAGES,
    mlp_grad_workspace_bytes,
    check_labels,
    device_info,
    clock_probe,
    sgemm,
    sgemm_flops,
    status_string,
    version,
)
