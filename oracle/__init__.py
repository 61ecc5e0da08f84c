"""CPU oracle for the routed-LoRA hot path.  Test infrastructure only: nothing in the
product package imports this."""
from .cpu_oracle import (route_gate, gate_logits, route_vocab, bucket, apply, apply_rows,
                         num_threads, expf, gelu, mlp_logits, topk_softmax, apply_mix,
                         route_compose)

__all__ = ["route_gate", "gate_logits", "route_vocab", "bucket", "apply", "apply_rows",
           "num_threads", "expf", "gelu", "mlp_logits", "topk_softmax", "apply_mix",
           "route_compose"]
