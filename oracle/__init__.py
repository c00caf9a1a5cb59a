"""CPU fp64 oracle for the Kunlun attention operators and SumKronLinear (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It shares no code with the HIP library and imports nothing from it.
"""
from .reference import (OracleLib, ACT_GELU, ACT_GELU_POLY, ACT_GELU_TANH, ACT_IDENTITY, ACT_RELU, ACT_SILU, ACT_SOFTMAX, act_deriv,
                        act_value, gdpa_bwd, gdpa_fwd, num_threads, seed_attn_bwd, seed_attn_fwd, sumkron_bwd, sumkron_fwd, swa_bwd, swa_fwd)

__all__ = ["OracleLib", "ACT_SOFTMAX", "ACT_IDENTITY", "ACT_RELU", "ACT_GELU", "ACT_GELU_TANH", "ACT_GELU_POLY", "ACT_SILU", "gdpa_fwd",
           "gdpa_bwd", "seed_attn_fwd", "seed_attn_bwd", "swa_fwd", "swa_bwd", "sumkron_fwd", "sumkron_bwd", "act_value", "act_deriv", "num_threads"]
