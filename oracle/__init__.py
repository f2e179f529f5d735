"""CPU oracle (test infrastructure).  See sd_oracle.c for what it follows.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package; the HIP library never does.
"""
from .binding import (  # noqa: F401
    OracleModel,
    OracleSeq,
    accept,
    argmax,
    build,
    cdf_distance,
    next_weights,
    rmsnorm,
    rope,
    round_bf16,
    route,
    sample_cdf,
    softmax_T,
)
from .metrics import acceptance_rate, alpha_hat, eq1_speedup, expected_tau, mean_tau  # noqa: F401
from .loop import StepRecord, ar_generate, prefill, sd_generate  # noqa: F401
