"""CPU oracle for batched rollout decoding (TEST INFRASTRUCTURE ONLY).

A plain, slow, obviously-correct NumPy implementation of what one rollout step
of the policy model computes: next-token samples, the per-token log-probabilities
that the trainer's importance ratios consume (paper Sec. 3.3, "field-based
storage": responses and log probabilities are per-sample fields; App. B.3), and,
for MoE policies, the per-token top-K expert indices recorded at every MoE layer
for Rollout Routing Replay (paper Sec. 5.5).

The paper delegates generation to an external inference engine and gives no
model equations; the arithmetic here is the standard decoder-only transformer
fixed by the workload shapes (RMSNorm eps 1e-6, rotary theta 1e6, GQA, SwiGLU,
top-8 softmax gating with renormalised weights, untied LM head).

Arithmetic is float32 by default (every function follows the dtype of its
inputs, so tests can also run it in float64); weights are bf16 bit patterns
upcast exactly.  The workloads fix the KV cache as bf16, so keys and values are
rounded to bf16 (nearest-even) once, when stored; everything else stays in the
working dtype.  The FP16 precision option (paper App. "FP16 vs. BF16 precision
ablation") replaces bf16 by IEEE fp16 in both places and nothing else.

Nothing in the product path may import this package: only tests/, the smoke
check and the benchmark's CPU-baseline leg use it.  It shares no code with the
HIP implementation.

Parity status: every function here is pinned by closed forms, brute force,
invariants or library routines in tests/test_oracle_*.py.  Agreement with a real
trained checkpoint of the named model family is *parity unpinned* (no such
checkpoint is available offline).
"""
from .layers import (rmsnorm, rope, attention, attention_bruteforce, silu, swiglu_ffn, moe_gate, moe_order_gap,
                     moe_ffn, moe_ffn_bruteforce, log_softmax)
from .philox import philox4x32_10, uniform_u32, gumbel_noise, sample_gumbel_max
from .model import OracleModel, forward_full, OracleRollout, round_to_bf16, round_to_f16

__all__ = ["rmsnorm", "rope", "attention", "attention_bruteforce", "silu", "swiglu_ffn", "moe_gate", "moe_order_gap",
           "moe_ffn", "moe_ffn_bruteforce", "log_softmax", "philox4x32_10", "uniform_u32", "gumbel_noise",
           "sample_gumbel_max", "OracleModel", "forward_full", "OracleRollout", "round_to_bf16", "round_to_f16"]
