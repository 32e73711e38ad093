"""CPU oracle of the MoE-layer forward pass -- test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the GPU library and its Python binding never do.
"""
from .moe_oracle import (ACT, OracleOut, build, capacity, combine, ffn_rows, gate_logits,
                         moe_layer, plan, scatter, threads, topk_softmax, act_value)

__all__ = ["ACT", "OracleOut", "build", "capacity", "combine", "ffn_rows", "gate_logits",
           "moe_layer", "plan", "scatter", "threads", "topk_softmax", "act_value"]
