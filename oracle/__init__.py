"""CPU oracle for the TriSpec verification pass.  TEST INFRASTRUCTURE ONLY.

Plain numpy, fp64, no blocking, no fusion: the definition written out so it
can be checked against the paper by eye.  Only tests, the smoke check and the
bench's cpu_baseline leg may import this package; the product path (the HIP
library and its Python binding) never does, and shares no code with it.

Pins (tests/test_oracle_*.py): brute-force sequential autoregressive forwards,
an independent torch-CPU forward, closed forms for RMSNorm / RoPE / softmax
statistics, the set-min definitions of tau_a and tau_m (paper Eq. 7, Eq. 9)
enumerated exhaustively, and the invariants at lambda = 0 and lambda > 1; for the
sampling form (Sec. 2.1, Eq. 6) the exactness of speculative sampling by enumeration
and by Monte Carlo, its greedy limit, and exact interval counts of the inverse CDF.
No function here is "parity unpinned".
"""
from .forward import (  # noqa: F401
    OracleWeights,
    bf16_round,
    rmsnorm,
    rope_angles,
    apply_rope,
    causal_forward,
    verify_forward,
    ancestor_sets,
    adapter,
)
from .decision import (  # noqa: F401
    CRIT_MARGIN,
    CRIT_TOP1,
    CRIT_ENTROPY,
    draft_ranks,
    node_stats,
    decide,
    chain_tau_a,
    chain_tau_m,
    chain_round_output,
    tie_flags,
    prune_reroot,
)
from .rounds import commit, greedy_decode, trispec_rounds, trispec_sample_rounds, verify_rounds  # noqa: F401
from .sampling import (  # noqa: F401
    RESAMPLE_DIRECT,
    RESAMPLE_RESIDUAL,
    accept_probability,
    inverse_cdf,
    residual_distribution,
    residual_mass,
    sample_decide,
    tempered_softmax,
)
