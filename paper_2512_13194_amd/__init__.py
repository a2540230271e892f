"""EARS verification step for AMD MI355X: Python binding of the HIP library.

`paper_2512_13194_amd.binding` mirrors the C ABI of include/ears.h name for name;
`paper_2512_13194_amd.sampler` wraps it in a verifier object for a decoding loop;
`paper_2512_13194_amd.inputs` draws the seeded synthetic workloads;
`paper_2512_13194_amd.build` compiles libears.so in-tree with hipcc.
"""
from .binding import (  # noqa: F401
    EARS_BF16,
    EARS_F32,
    EARS_NOALLOC_SCRATCH_BYTES,
    EARS_NSTATS,
    EARS_OK,
    EARS_STAGE_ALL,
    EARS_STAGE_DECIDE,
    EARS_STAGE_SAMPLE,
    EARS_STAGE_STATS,
    EARS_UNCERTAINTY_ENTROPY,
    EARS_UNCERTAINTY_MAXPROB,
    EARS_UNCERTAINTY_VARIANCE,
    STAT_NAMES,
    EarsError,
    ears_bench_copy,
    ears_bench_read,
    ears_test_single_launch,
    ears_greedy_workspace_bytes,
    ears_import_stats,
    ears_lm_head_bf16,
    ears_lm_head_workspace_bytes,
    ears_release,
    ears_row_stats,
    ears_verify_bf16,
    ears_verify_ex,
    ears_verify_f32,
    ears_verify_greedy,
    ears_verify_noalloc,
    ears_verify_ragged_bf16,
    ears_verify_ragged_f32,
    ears_workspace_bytes,
    lib,
    status_string,
)
from .sampler import EarsVerifier, VerifyResult, acceptance_sweep  # noqa: F401,E402
