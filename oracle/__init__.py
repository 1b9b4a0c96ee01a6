"""fp64 CPU oracle for AdamA -- test infrastructure only.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package; the product package never does.
"""
from .adama_oracle import (  # noqa: F401
    OracleState,
    alg1_step,
    apply,
    apply_adamw,
    begin_step,
    bf16_to_f64,
    build,
    ddp_combine,
    f16_to_f64,
    fold,
    fold_scaled,
    lib_path,
    sgdm_apply,
    sgdm_begin_step,
    sgdm_fold,
    widen,
)
