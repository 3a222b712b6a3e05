"""MI355X-native Lightning Attention-2 hot path (gfx950 HIP kernels behind a C ABI)."""
from .binding import (  # noqa: F401
    LA2Error,
    lib_path,
    load,
    la2_fwd,
    la2_bwd,
    la2_fwd_state,
    la2_bwd_state,
    la2_fwd_norm,
    la2_fwd_varlen,
    la2_bwd_varlen,
    la2_bwd_norm,
    la2_decode_step,
    la2_decode_multi,
    la2_left_product_fwd,
    la2_stream_probe,
    la2_workspace_bytes,
)
