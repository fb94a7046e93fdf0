"""Seeded synthetic inputs shared by the oracle-side tests and the device-side
tests/benchmark.  Holds no arithmetic of the verification method itself: only
shapes, random draws and storage-type casts done by library routines."""
from .configs import CONFIGS, Shape, scaled_down  # noqa: F401
from .synth import (make_weights, make_prefix_lengths, make_tokens, make_uniforms,  # noqa: F401
                    make_kv_block, make_random_q, sample_from, weights_to_numpy)
