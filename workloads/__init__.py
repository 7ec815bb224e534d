"""Seeded synthetic inputs shaped like the paper's workloads.

This package serves both the GPU library's tests/benchmark and the CPU oracle's tests.
It contains no arithmetic of the method (no sign, momentum, vote or update): it only
draws random tensors, and -- for the pre-packed vote stress input and the random-sign
adversary -- random bit patterns.  Everything is generated with torch generators on the
requested device; GPU-side tests copy what they generated to the host and hand the same
bytes to the oracle, so the two sides never depend on matching random number streams.

Workloads (sizes as in the paper's experiments, Section 4, and in this build's five
configurations; "N(0, s)" is read as standard deviation s):
  tiny       d = 65,536,      M = 3   N(0,1) fp32 gradients, weights N(0, 0.02)
  resnet50   d = 25,557,032,  M = 15  g_m = mu + N(0, 1e-2), mu ~ N(0, 1e-3) fixed per run;
                                      seed of worker m at step k = base + 1000*k + m
  adversary  same shape; workers 0..6 invert or randomise their transmitted signs
  stress     d = 2**30,       M = 255 pre-packed bits, bit ~ Bernoulli(p_j), p_j ~ U(0.3, 0.7)
  large      d = 1.5e9,       M = 31  bf16 gradients and weights, same signal/noise recipe
"""
from .generators import (  # noqa: F401
    RESNET50_D,
    LARGE_D,
    STRESS_D,
    gaussian,
    tiny_config,
    shared_mean,
    worker_gradients,
    random_words,
    resnet50_parameter_shapes,
    bernoulli_packed_rows,
    special_values_f32,
    words_for,
    to_numpy,
    bf16_bits,
)
