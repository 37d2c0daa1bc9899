"""CPU oracle for the GuidedQuant Fisher-Gram path (test infrastructure only).

Nothing in the product package may import this module: only the tests, the
smoke check and the benchmark's cpu_baseline leg call it.
"""
from .gq_oracle import (  # noqa: F401
    group_partition,
    group_weights,
    fisher_gram,
    fisher_gram_block,
    objective,
    per_channel_hessian,
    unaveraged_objective,
    objective_from_tokens,
    objective_rows_from_tokens,
    cd_coordinate_target,
    cd_assign,
    lnq_codebook,
    lnq,
    damped_cholesky,
    gptq_assign,
    ldlq_assign,
)
