"""CPU oracle for the batched MPE simple-spread rollout.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The product package never imports this.
"""
from .mpe_oracle import Oracle, OracleConfig, build, philox4x32_10, gumbel_max_action, uniform_action, round_to_bf16, log_probs  # noqa: F401
