"""libadama: the AdamA (Adam Accumulation) optimizer hot path for AMD MI355X (gfx950).

`binding` mirrors the C ABI declared in include/adama.h; `harness` is the simulated
backward pass that feeds it per-layer gradients from a single reusable buffer.
"""
from .binding import (  # noqa: F401
    AdamaError,
    adama_apply,
    adama_apply_multi,
    adama_begin_step,
    adama_begin_step_multi,
    adama_fold,
    adama_fold_first,
    adama_fold_first_multi,
    adama_fold_last_apply,
    adama_fold_last_apply_multi,
    adama_fold_multi,
    adama_last_error,
    adama_max_tensors_per_launch,
    adama_rescale_apply,
    adama_rescale_apply_multi,
)
