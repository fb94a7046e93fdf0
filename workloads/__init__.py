"""Seeded synthetic inputs shared by the oracle-side tests and the device-side
tests/benchmark.  Holds no arithmetic of the verification method itself: only
shapes, random draws and storage-type casts done by library routines.
`device_case`, `profile_plan` and `profile_prefill` (not imported here) set these workloads up on the GPU
through the library's binding, for the benchmark, the full-size tests and the profiling drivers."""
from .configs import CONFIGS, Shape, scaled_down  # noqa: F401
from .synth import (make_weights, make_prefix_lengths, make_tokens, make_uniforms,  # noqa: F401
                    make_kv_block, make_random_q, sample_from, weights_to_numpy)
