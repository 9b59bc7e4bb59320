"""Float64 CPU oracle for the ATP hot path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this package: only `tests/`,
`__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` do.
It shares no code with the HIP path.
"""
from .atp_oracle import (  # noqa: F401
    qf,
    principal_bases,
    lowrank_linear,
    attention,
    linearised_attention,
    rope,
    project_onto_bases,
    rope_principal_keys,
    dense_attention_layer,
    atp_layer,
    concat_factors,
    norm_factored,
    atp_block,
    rayleigh_ritz,
    alternating_rank1,
    svd_entropy,
)
