"""MI355X-native Visual Perception Engine hot path: thin Python binding over libvpe.so.

The library (HIP, gfx950) does all the computing; this package only marshals arguments.
PyTorch-ROCm supplies device memory and streams.
"""
from .binding import (  # noqa: F401
    Engine, HeadCfg, VpeError, lib, load_library,
    vpe_create, vpe_destroy, vpe_encode, vpe_encode_at, vpe_feat_view, vpe_preprocess_u8, vpe_next_encode_stream, preprocess_u8, vpe_head_output, vpe_last_error, vpe_run_head,
    vpe_run_head_latest, vpe_run_head_static, vpe_head_counters, vpe_frame_ready,
    vpe_set_head_rate, vpe_set_head_rate_hz, vpe_stats, vpe_sync, vpe_head_done, vpe_wait_head, vpe_stage_times, vpe_time_kernel, vpe_workspace_bytes,
    VPE_OK, VPE_SKIPPED, VPE_BUSY, VPE_EINVAL, VPE_ENOMEM, VPE_ESTALE, VPE_EHIP,
    VPE_F32, VPE_BF16, VPE_MLP_GELU, VPE_MLP_SWIGLU, VPE_HEAD_SEG, VPE_HEAD_DEPTH, VPE_HEAD_DET, VPE_HEAD_DPT,
    VPE_FLAG_GRAPHS, VPE_FLAG_HOST_ONLY, VPE_FLAG_WALL_CLOCK, VPE_FLAG_TIMING,
)
