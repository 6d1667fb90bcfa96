"""CPU oracle for the speculative draft-and-verify decode step.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package; the product
path never does.  It shares no code with the HIP library.
"""
from .model import OracleModel, build_oracle, round_storage  # noqa: F401
from .sd import (  # noqa: F401
    SpecDecoder, plain_decode, accept_greedy, accept_sample, softmax64, inv_cdf, argmax_f32,
    expected_tokens_per_step, projected_speedup,
)
