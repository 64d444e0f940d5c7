"""MI355X-native forward kernels for the Hyena-SE / Hyena-MR gated causal convolutions.

``binding`` exposes the C ABI of ``libhyena.so`` under the same names; ``synth`` draws the seeded
benchmark inputs; ``build`` compiles the library.
"""
from .binding import (  # noqa: F401
    HyenaError,
    Plan,
    plan_bwd,
    plan_bwd_shard,
    plan_chain,
    plan_featurize3,
    plan_gated,
    plan_gated_shard,
    plan_li,
    hyena_chain_fwd,
    hyena_chain_fwd_shard,
    hyena_featurize3_fwd,
    hyena_featurize_fwd,
    hyena_li_fwd,
    hyena_li_fwd_static,
    hyena_li_fwd_carry,
    hyena_mr_bwd,
    hyena_mr_bwd_shard,
    hyena_mr_fwd,
    hyena_mr_fwd_shard,
    hyena_se_bwd,
    hyena_se_bwd_shard,
    hyena_se_fwd,
    hyena_se_fwd_shard,
    hyena_stream_copy,
    hyena_stream_gate,
    plan_stream_gate,
    set_option,
    status_string,
    version,
)
