"""fp64 CPU oracle for Lightning Attention-2 (test infrastructure only).

Only the tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It shares no code with the GPU library and never imports it.
"""
from .ref import (  # noqa: F401
    build,
    num_threads,
    fwd_direct,
    bwd_direct,
    fwd_recurrent,
    bwd_recurrent,
    bwd_recurrent_state,
    decode_step,
    fwd_rows,
    bwd_rows,
)
from .block_form import block_forward, block_backward, state_update_residuals  # noqa: F401
from .norm import (  # noqa: F401
    fwd_norm, bwd_norm, norm_backward_rows, fwd_norm_state, bwd_norm_state, fwd_norm_packed, bwd_norm_packed,
)
