"""Seeded synthetic inputs (gradient and weight values, workload shapes) for tests and benchmarks."""
from . import configs, gen  # noqa: F401
from .gen import Spec, fill_device, fill_host, stream_key, widen  # noqa: F401
