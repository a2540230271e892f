"""CPU oracle for the EARS verification step.  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may import this package;
the GPU library never does, and the two share no code.
"""
from .ears_oracle import (  # noqa: F401
    NDIAG,
    NSAMP,
    OracleResult,
    UNC_ENTROPY,
    UNC_MAXPROB,
    UNC_VARIANCE,
    entropy,
    variance,
    accept_uniform,
    build,
    gumbel,
    gumbel_uniform,
    lm_head,
    lm_head_dot,
    round_bf16,
    philox4x32_10,
    softmax,
    top2,
    verify,
    verify_greedy,
    verify_ragged,
)
