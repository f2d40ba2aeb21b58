"""FP64 CPU oracle for the 1D dilated convolution layer (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It shares nothing with the HIP path and imports nothing from it.
"""
from .conv1d_oracle import (  # noqa: F401
    build,
    out_width,
    threads,
    fwd,
    bwd_data,
    bwd_weight,
    fwd_at,
    bwd_data_at,
    bwd_weight_at,
    round_bf16,
    epilogue,
    fwd_ex,
    bwd_data_ex,
)
