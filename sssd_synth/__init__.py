"""Seeded synthetic inputs for the SSSD verification step.

This module serves BOTH the CPU oracle and the HIP path and therefore holds
none of the method's arithmetic: it only turns (seed, tensor id, element index)
into numbers.  Everything is computed with wrapping 64-bit integer arithmetic
plus one exact int->float scale, so a tensor generated on the CPU and the same
tensor generated on a GPU by torch are bit-identical.

Recipe
------
* counter-based hash: splitmix64 finaliser applied to
  ``key(seed, tensor_id) + counter * GOLDEN`` (all mod 2**64);
* "normal" values: centred Irwin-Hall sum of eight 16-bit uniform fields taken
  from two consecutive hashes, scaled to the requested standard deviation
  (variance matched exactly; excess kurtosis -0.15; support +-4.9 sigma), then
  rounded fp64 -> fp32 -> bf16 (round-to-nearest-even);
* uniform integers: ``hash mod range`` on the non-negative 63-bit hash.
"""
from .gen import (  # noqa: F401
    TensorId,
    hash_u64_python,
    normal_bf16,
    uniform_int,
    uniform_bf16,
    repetitive_stream,
    ModelShape,
    MODEL_SHAPES,
    layer_weight_specs,
    global_weight_specs,
    make_weight,
    make_kv_prefill,
)
